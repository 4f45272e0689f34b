// Recovery profile (paper Section 2.4, at block granularity): the attention weight every
// query block puts on every key block of the causal triangle, under full attention.
//
//   mass[s][h][i][j] = 1/n_i * sum over the valid queries t of block i, keys u of block j, u <= t,
//                      of softmax_t(q_t . k_u * scale)                    (j <= i; rows sum to 1)
//
// This is the offline profiling step: sorted per row and accumulated it gives the recovery
// curves that budget shifting consumes, and summed over a selection it says how much of the
// attention that selection keeps.  It is a dense pass and not on the hot path; it shares the
// first contraction of the attention kernels (64-key K tiles copied global->LDS into swizzled
// 256-byte rows, S^T = K Q^T with Q in registers, a lane owns one query column) and has no
// second one.
//
// One workgroup = one (sequence, head, query block) row, all key blocks 0 .. i, in two sweeps:
//   sweep A: per lane, the exact running maximum and sum of exp2 over its share of the keys
//            (fp32, nothing rounded to bf16), merged with the lane that holds the other half of
//            the query's keys: log2 of the softmax denominator per query, kept in registers;
//   sweep B: the scores again, probabilities exp2(s - lse), summed over the lane's keys, the
//            tiles of a key block, the wave (shuffles) and the waves (LDS, fixed order):
//            one number per key block.
// Rows are launched heaviest first (largest i first), so the tail of the launch is short rows.
#include "attn_common.h"

namespace shplb {
namespace {

template <int BQ>
__global__ __launch_bounds__(2 * BQ) void mass_kernel(SeqMeta meta, Strides st, const uint16_t* __restrict__ q,
                                                      const uint16_t* __restrict__ k, float* __restrict__ mass,
                                                      int max_nb, float scale_log2) {
  constexpr int kWaves = BQ / 32;
  constexpr int SUB = BQ / kKeysPerTile;            // 64-key tiles per key block
  constexpr int kRoundRows = 4 * kWaves;
  constexpr int kRounds = kKeysPerTile / kRoundRows;

  __shared__ __attribute__((aligned(1024))) char k_lds[2][kTileBytes];
  __shared__ float s_part[2][kWaves];

  // blockIdx.x = level * (sequences * heads) + (s * heads + h); level 0 is the last query block
  const int per_level = meta.n_seq * meta.n_q_heads;
  const int level = blockIdx.x / per_level, sh = blockIdx.x - level * per_level;
  const int s = sh / meta.n_q_heads, h = sh - s * meta.n_q_heads;
  const int nb = meta.blk_begin[s + 1] - meta.blk_begin[s];
  const int i = max_nb - 1 - level;
  if (i >= nb) return;                              // shorter sequence of a varlen batch

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hi = lane >> 5;
  const int g = kv_head_of(meta, h);
  const int seq_begin = meta.tok_begin[s], seq_end = meta.tok_begin[s + 1];
  const int n_tiles = (i + 1) * SUB;
  const int64_t row_bytes = st.kv_t * 2;
  const char* k_head = reinterpret_cast<const char*>(k + int64_t(g) * st.kv_h);

  const int cp_row = 4 * wave + (lane >> 4);
  const int k_rd0 = n * kRowBytes + ((hi ^ swz(n)) << 4);
  const uint32_t k_stage0 = __builtin_amdgcn_readfirstlane(lds_offset_of(&k_lds[0][0]) + 4 * wave * kRowBytes);

  // Copy the 64 keys of tile `it` (block it / SUB) into LDS stage `buf`.
  auto issue_tile = [&](int it, int buf) {
    const int j = it / SUB, sub = it - j * SUB;
    // a tile that starts past the end of a ragged last block is moved back onto the last token
    const int key_base = min(seq_begin + j * BQ + kKeysPerTile * sub, seq_end - 1);
    const int last = seq_end - 1 - key_base;
    const char* k_tile = k_head + int64_t(key_base) * row_bytes;
#pragma unroll
    for (int rd = 0; rd < kRounds; ++rd) {
      const int r = rd * kRoundRows + cp_row;
      // rows past the end of the sequence re-read the last valid key; they are masked
      const uint32_t off = uint32_t(min(r, last)) * uint32_t(row_bytes) + (((lane & 15) ^ swz(r)) << 4);
      copy_g2l_16(k_tile, off, k_stage0 + buf * kTileBytes + rd * kRoundRows * kRowBytes);
    }
  };
  issue_tile(0, 0);

  // Q fragments: B operand of S^T = K Q^T, lane (n, hi) holds dims 16ks + 8hi.. of its query
  bf16x8 qf[8];
  const int q_tok = seq_begin + i * BQ + wave * 32 + n;
  {
    const uint16_t* src = q + int64_t(min(q_tok, seq_end - 1)) * st.q_t + int64_t(h) * st.q_h + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
  }
  const int n_valid = min(BQ, seq_end - seq_begin - i * BQ);
  float* out_row = mass + meta.score_off[s] + (int64_t(h) * nb + i) * nb;

  // raw scores (q . k, unscaled) of tile `it` from stage `buf`; on the diagonal block the keys above the
  // query are set to -inf (only there: the test is uniform, so other tiles pay nothing for it)
  auto scores_of = [&](int it, int buf, f32x16 (&sc)[2]) {
    const char* kt = k_lds[buf];
    bf16x8 kf[2][8];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        kf[mt][ks] = *reinterpret_cast<const bf16x8*>(kt + (k_rd0 ^ (ks << 5)) + mt * 32 * kRowBytes);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[mt][r] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
        sc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][ks], qf[ks], sc[mt], 0, 0, 0);
    const int j = it / SUB, sub = it - j * SUB;
    if (j == i) {
      int d = kKeysPerTile * sub + 4 * hi - (wave * 32 + n);      // key position minus query position, per register below
      asm volatile("" : "+v"(d));                                  // keep the 32 comparisons here, not hoisted as masks
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (d + (32 * mt + 8 * (r >> 2) + (r & 3)) > 0) sc[mt][r] = -INFINITY;
    }
  };

  // ---- sweep A: log2 of the softmax denominator of the lane's query.  The sum runs against a reference
  // exponent that is only raised when a tile's maximum exceeds it by more than 2^8 (then the sum so far
  // is rescaled): exact in real arithmetic, and most tiles cost one fused multiply-add, one exponential
  // and one addition per score, plus the maximum.
  float m_run = -INFINITY, l_run = 0.0f;
  int step = 0;                                     // tiles handled so far over both sweeps: stage = step & 1
  for (int it = 0; it < n_tiles; ++it, ++step) {
    wait_vmem_all();
    __syncthreads();
    issue_tile(it + 1 < n_tiles ? it + 1 : 0, (step + 1) & 1);           // the last one starts sweep B
    f32x16 sc[2];
    scores_of(it, step & 1, sc);
    float mx = fmaxf(sc[0][0], sc[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(sc[0][r], sc[1][r]));
    mx *= scale_log2;
    if (mx > m_run + kRescaleSlack) {               // per lane: a lane's reference follows its own keys
      l_run *= m_run == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(m_run - mx);
      m_run = mx;
    }
    if (m_run != -INFINITY) {                       // all keys of the lane masked so far: nothing to add
      float sum0 = 0.0f, sum1 = 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        sum0 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0][r], scale_log2, -m_run));
        sum1 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[1][r], scale_log2, -m_run));
      }
      l_run += sum0 + sum1;
    }
  }
  float lse2;
  {
    float m_lo, m_hi, l_lo, l_hi;                   // the two lanes of a query hold disjoint halves of its keys
    pair_values(m_run, m_lo, m_hi);
    pair_values(l_run, l_lo, l_hi);
    const float m_all = fmaxf(m_lo, m_hi);
    const float l_all = (m_lo == -INFINITY ? 0.0f : l_lo * __builtin_amdgcn_exp2f(m_lo - m_all)) +
                        (m_hi == -INFINITY ? 0.0f : l_hi * __builtin_amdgcn_exp2f(m_hi - m_all));
    lse2 = m_all + __builtin_amdgcn_logf(l_all);    // v_log_f32 is a base-2 logarithm
  }
  const bool live = q_tok < seq_end;                // padding queries of a ragged last block count nothing

  // ---- sweep B: probabilities, summed per key block
  float acc = 0.0f;
  for (int it = 0; it < n_tiles; ++it, ++step) {
    wait_vmem_all();
    __syncthreads();
    if (it + 1 < n_tiles) issue_tile(it + 1, (step + 1) & 1);
    const int j = it / SUB, sub = it - j * SUB;
    if (sub == 0 && j > 0 && tid == 0) {            // block j-1 is complete and visible: fixed-order sum
      float tot = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) tot += s_part[(j - 1) & 1][w];
      out_row[j - 1] = tot / float(n_valid);
    }
    f32x16 sc[2];
    scores_of(it, step & 1, sc);
    float sum0 = 0.0f, sum1 = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sum0 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0][r], scale_log2, -lse2));
      sum1 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[1][r], scale_log2, -lse2));
    }
    acc += live ? sum0 + sum1 : 0.0f;
    if (sub == SUB - 1) {
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d);
      if (lane == 0) s_part[j & 1][wave] = acc;
      acc = 0.0f;
    }
  }
  __syncthreads();
  if (tid == 0) {
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) tot += s_part[i & 1][w];
    out_row[i] = tot / float(n_valid);
  }
}

}  // namespace

int32_t launch_block_mass(const Geometry& g, const void* q, const void* k, float* mass, hipStream_t stream) {
  const SeqMeta& m = g.meta;
  const int64_t n_wg = int64_t(g.max_nb) * m.n_seq * m.n_q_heads;
  if (n_wg > 0x7fffffff) return SHPLB_E_UNSUPPORTED;
  const float scale_log2 = g.scale * 1.4426950408889634f;
  if (m.block == 128)
    hipLaunchKernelGGL((mass_kernel<128>), dim3(uint32_t(n_wg)), dim3(256), 0, stream, m, g.st,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), mass, g.max_nb, scale_log2);
  else
    hipLaunchKernelGGL((mass_kernel<64>), dim3(uint32_t(n_wg)), dim3(128), 0, stream, m, g.st,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), mass, g.max_nb, scale_log2);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
