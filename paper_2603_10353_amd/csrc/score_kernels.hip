// Block importance: mean-pool query/key blocks (HBM-bound streaming reduction), then
// pooled logits for the causal lower triangle (small fp32 MFMA contraction).
#include "shplb_internal.h"

namespace shplb {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

namespace {

constexpr int kPoolThreads = 256;
constexpr int kPoolWaves = 4;
constexpr int kPoolElems = 512;   // bf16 elements of a token row covered by one workgroup

__device__ __forceinline__ void add_bf16x8(float (&acc)[8], const u32x4 w) {
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    acc[2 * c] += __uint_as_float(w[c] << 16);
    acc[2 * c + 1] += __uint_as_float(w[c] & 0xffff0000u);
  }
}

// One workgroup = one block of tokens x 512 consecutive (head, dim) elements.
// The four waves take every fourth token; each lane owns 8 consecutive dims and
// keeps fp32 sums; partial sums meet in LDS in a fixed order (deterministic).
// blockIdx.x enumerates first the Q tiles, then the K tiles.
__global__ __launch_bounds__(kPoolThreads) void pool_kernel(
    SeqMeta meta, Strides st, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    float* __restrict__ qbar, float* __restrict__ kbar, int q_chunks, int k_chunks, int total_blocks) {
  __shared__ float part[kPoolWaves][kPoolElems];
  int bid = blockIdx.x;
  const bool is_q = bid < total_blocks * q_chunks;
  if (!is_q) bid -= total_blocks * q_chunks;
  const int chunks = is_q ? q_chunks : k_chunks;
  const int gblk = bid / chunks;
  const int chunk = bid - gblk * chunks;
  const int n_heads = is_q ? meta.n_q_heads : meta.n_kv_heads;
  const uint16_t* src = is_q ? q : k;
  const int64_t stride_t = is_q ? st.q_t : st.kv_t;
  const int64_t stride_h = is_q ? st.q_h : st.kv_h;
  float* dst = is_q ? qbar : kbar;

  int s = 0;
  while (s + 1 < meta.n_seq && gblk >= meta.blk_begin[s + 1]) ++s;
  const int t0 = meta.tok_begin[s] + (gblk - meta.blk_begin[s]) * meta.block;
  const int t1 = min(meta.tok_begin[s + 1], t0 + meta.block);
  const int cnt = t1 - t0;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e = chunk * kPoolElems + lane * 8;          // element inside the [heads*128] token row
  const int head = e >> 7, dim = e & 127;
  const bool live = head < n_heads;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (live) {
    const uint16_t* base = src + head * stride_h + dim;
    int t = t0 + wave;
    for (; t + 7 * kPoolWaves < t1; t += 8 * kPoolWaves) {
      u32x4 w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + int64_t(t + u * kPoolWaves) * stride_t));
#pragma unroll
      for (int u = 0; u < 8; ++u) add_bf16x8(acc, w[u]);
    }
    for (; t < t1; t += kPoolWaves) {
      const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + int64_t(t) * stride_t));
      add_bf16x8(acc, w);
    }
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) part[wave][lane * 8 + c] = acc[c];
  __syncthreads();
  for (int x = threadIdx.x; x < kPoolElems; x += kPoolThreads) {
    const int ee = chunk * kPoolElems + x;
    const int hh = ee >> 7, dd = ee & 127;
    if (hh < n_heads) {
      const float sum = ((part[0][x] + part[1][x]) + part[2][x]) + part[3][x];
      dst[(int64_t(hh) * total_blocks + gblk) * kHeadDim + dd] = sum / float(cnt);
    }
  }
}

// scores[s][h][i][j] = (qbar[h][i] . kbar[h/G][j]) * scale for j <= i.
// One workgroup = a 64x64 tile of one (sequence, head); each wave a 32x32 tile
// through v_mfma_f32_32x32x2_f32.  Operand slot k of a lane is dim 8c+4*(lane/32)+u,
// the same for both operands, so each lane reads 16-byte pieces of a pooled row.
__global__ __launch_bounds__(256) void score_kernel(
    SeqMeta meta, const float* __restrict__ qbar, const float* __restrict__ kbar,
    float* __restrict__ scores, int total_blocks, float scale) {
  const int sh = blockIdx.z;
  const int s = sh / meta.n_q_heads, h = sh - s * meta.n_q_heads;
  const int nb = meta.blk_begin[s + 1] - meta.blk_begin[s];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i0 = blockIdx.y * 64 + (wave >> 1) * 32;
  const int j0 = blockIdx.x * 64 + (wave & 1) * 32;
  if (i0 >= nb || j0 >= nb || j0 > i0 + 31) return;
  const int g = h / (meta.n_q_heads / meta.n_kv_heads);
  const int n = lane & 31, hi = lane >> 5;
  const int ia = min(i0 + n, nb - 1), jb = min(j0 + n, nb - 1);
  const float* a = qbar + (int64_t(h) * total_blocks + meta.blk_begin[s] + ia) * kHeadDim + 4 * hi;
  const float* b = kbar + (int64_t(g) * total_blocks + meta.blk_begin[s] + jb) * kHeadDim + 4 * hi;
  f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 4
  for (int c = 0; c < kHeadDim / 8; ++c) {
    const f32x4 av = *reinterpret_cast<const f32x4*>(a + 8 * c);
    const f32x4 bv = *reinterpret_cast<const f32x4*>(b + 8 * c);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], acc, 0, 0, 0);
  }
  float* out = scores + meta.score_off[s] + int64_t(h) * nb * nb;
  const int j = j0 + n;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = i0 + 8 * (r >> 2) + 4 * hi + (r & 3);
    if (i < nb && j <= i) out[int64_t(i) * nb + j] = acc[r] * scale;
  }
}

}  // namespace

int32_t launch_pool_scores(const Geometry& g, const void* q, const void* k, float* scores,
                           float* qbar, float* kbar, hipStream_t stream) {
  const SeqMeta& m = g.meta;
  const int q_chunks = (m.n_q_heads * kHeadDim + kPoolElems - 1) / kPoolElems;
  const int k_chunks = (m.n_kv_heads * kHeadDim + kPoolElems - 1) / kPoolElems;
  const int64_t n_wg = g.total_blocks * (q_chunks + k_chunks);
  if (n_wg > 0x7fffffff) return SHPLB_E_UNSUPPORTED;
  hipLaunchKernelGGL(pool_kernel, dim3(uint32_t(n_wg)), dim3(kPoolThreads), 0, stream, m, g.st,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), qbar, kbar,
                     q_chunks, k_chunks, int(g.total_blocks));
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  const int tiles = (g.max_nb + 63) / 64;
  hipLaunchKernelGGL(score_kernel, dim3(tiles, tiles, m.n_seq * m.n_q_heads), dim3(256), 0, stream, m,
                     qbar, kbar, scores, int(g.total_blocks), g.scale);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
