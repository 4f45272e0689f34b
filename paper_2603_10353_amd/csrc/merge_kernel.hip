// Merge of the pieces of rows that were split along their selected key blocks.
//
// A piece c of a row leaves, per query, what the attention kernel holds when it has seen the
// piece's keys: the unnormalised output O_c, the sum l_c of its probabilities, both relative
// to a reference exponent m_c (p = 2^(s*scale*log2e - m_c)).  Softmax over the union of the
// pieces (Eq. 1 over the selected keys) is then, with m = max_c m_c and w_c = 2^(m_c - m),
//
//     out = sum_c w_c O_c / sum_c w_c l_c,      lse = (m + log2 sum_c w_c l_c) ln 2,
//
// summed in piece order, so the result does not depend on which workgroup computed which
// piece or on the slot numbers.  One workgroup per split row; launched over the largest
// number of rows that can be split, workgroups past the count return at once.
#include "attn_common.h"

namespace shplb {
namespace {

constexpr int kMergeThreads = 256;

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(SeqMeta meta, Strides st, SplitBuffers sb,
                                                              uint16_t* __restrict__ out, float* __restrict__ lse,
                                                              int64_t total_tokens) {
  if (blockIdx.x >= sb.count->n_rows) return;
  const SplitRow sr = sb.rows[blockIdx.x];
  if (sr.pieces < 2 || sr.slot < 0 || sr.slot + sr.pieces > sb.slot_capacity) return;
  int s, h, i, nb;
  decode_row(meta, sr.row, s, h, i, nb);
  const int seq_begin = meta.tok_begin[s], seq_end = meta.tok_begin[s + 1];
  const float* part_o = sb.part_o + int64_t(sr.slot) * kSlotFloatsO;
  const float* part_ml = sb.part_ml + int64_t(sr.slot) * kSlotFloatsML;

  // a thread owns four consecutive dims of one query; 32 threads cover a query's 128 dims
  for (int e = threadIdx.x; e < 128 * (kHeadDim / 4); e += kMergeThreads) {
    const int q_in = e / (kHeadDim / 4), d = 4 * (e - q_in * (kHeadDim / 4));
    const int q_tok = seq_begin + i * 128 + q_in;
    if (q_tok >= seq_end) continue;                 // padding of a ragged last block
    float m = -INFINITY;
    for (int c = 0; c < sr.pieces; ++c) m = fmaxf(m, part_ml[c * kSlotFloatsML + q_in]);
    float l = 0.0f;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int c = 0; c < sr.pieces; ++c) {
      const float m_c = part_ml[c * kSlotFloatsML + q_in];
      const float w = m_c == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(m_c - m);
      l += w * part_ml[c * kSlotFloatsML + 128 + q_in];
      const f32x4 o = *reinterpret_cast<const f32x4*>(part_o + c * kSlotFloatsO + q_in * kHeadDim + d);
      acc += w * o;
    }
    const float inv = 1.0f / l;
    u32x2 w2;
    w2.x = pack_bf16(acc.x * inv, acc.y * inv);
    w2.y = pack_bf16(acc.z * inv, acc.w * inv);
    *reinterpret_cast<u32x2*>(out + int64_t(q_tok) * st.q_t + int64_t(h) * st.q_h + d) = w2;
    if (lse != nullptr && d == 0)
      lse[int64_t(h) * total_tokens + q_tok] = (m + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
  }
}

}  // namespace

int32_t launch_merge(const Geometry& g, SplitBuffers sb, void* out, float* lse, hipStream_t stream) {
  const int n_wg = sb.slot_capacity / 2;            // a split row has at least two pieces
  if (n_wg < 1) return SHPLB_OK;
  hipLaunchKernelGGL(merge_kernel, dim3(n_wg), dim3(kMergeThreads), 0, stream, g.meta, g.st, sb,
                     static_cast<uint16_t*>(out), lse, g.total_tokens);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
