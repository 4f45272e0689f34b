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
// One workgroup = a 128x128 tile of one (sequence, head); each wave a 64x64 tile as
// 2x2 MFMA tiles of v_mfma_f32_32x32x2_f32.  The pooled rows are staged through LDS in
// eight slices of 16 dims (coalesced 16-byte loads, 80-byte padded rows: conflict-free
// 16-byte operand reads); five or more workgroups fit a compute unit (all tiles of a 128K layer are resident at once), so some load while
// others multiply.  Operand slot k of a lane is dim 8c + 4*(lane/32) + u, the same
// for both operands.  Every output accumulates over dims in ascending (half, c, u)
// order: results are deterministic and independent of the tiling.
constexpr int kScoreTile = 128;
constexpr int kScoreHalf = 16;
constexpr int kScoreRow = kScoreHalf + 4;   // floats per LDS row

__global__ __launch_bounds__(256) void score_kernel(
    SeqMeta meta, const float* __restrict__ qbar, const float* __restrict__ kbar,
    float* __restrict__ scores, int total_blocks, float scale) {
  __shared__ __attribute__((aligned(16))) float a_lds[kScoreTile * kScoreRow];
  __shared__ __attribute__((aligned(16))) float b_lds[kScoreTile * kScoreRow];
  const int sh = blockIdx.z;
  const int s = sh / meta.n_q_heads, h = sh - s * meta.n_q_heads;
  const int nb = meta.blk_begin[s + 1] - meta.blk_begin[s];
  // blockIdx.x enumerates only the tiles of the lower triangle (row-major: tile row r holds
  // tiles r(r+1)/2 .. r(r+1)/2 + r).  Consecutive workgroup ids go to different XCDs, so
  // every die gets the same share of live tiles (a square grid would hand die x the whole
  // tile column x, 8 tiles for column 0 against 1 for column 7).
  int tr = int((__builtin_sqrtf(8.0f * float(blockIdx.x) + 1.0f) - 1.0f) * 0.5f);
  while (tr * (tr + 1) / 2 > int(blockIdx.x)) --tr;
  while ((tr + 1) * (tr + 2) / 2 <= int(blockIdx.x)) ++tr;
  const int ti = tr * kScoreTile, tj = (int(blockIdx.x) - tr * (tr + 1) / 2) * kScoreTile;
  if (ti >= nb) return;                             // shorter sequence of a varlen batch
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int i0 = ti + 64 * wi, j0 = tj + 64 * wj;
  const bool active = i0 < nb && j0 < nb && j0 <= i0 + 63;   // this wave's tile touches the triangle
  const int g = h / (meta.n_q_heads / meta.n_kv_heads);
  const int n = lane & 31, hi = lane >> 5;
  const float* a_rows = qbar + (int64_t(h) * total_blocks + meta.blk_begin[s]) * kHeadDim;
  const float* b_rows = kbar + (int64_t(g) * total_blocks + meta.blk_begin[s]) * kHeadDim;

  f32x16 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.0f;

  constexpr int kSlices = kHeadDim / kScoreHalf;
  constexpr int kPieces = kScoreHalf / 4;           // 16-byte pieces per staged row
  constexpr int kLoads = kScoreTile * kPieces / 256; // pieces per thread, for A and for B
  f32x4 va[kLoads], vb[kLoads];
  auto fetch = [&](int half) {                      // global -> registers, one slice ahead of its use
#pragma unroll
    for (int x = 0; x < kLoads; ++x) {
      const int idx = tid + 256 * x;
      const int row = idx / kPieces, piece = idx % kPieces;
      const int ia = min(ti + row, nb - 1), jb = min(tj + row, nb - 1);
      va[x] = *reinterpret_cast<const f32x4*>(a_rows + int64_t(ia) * kHeadDim + kScoreHalf * half + 4 * piece);
      vb[x] = *reinterpret_cast<const f32x4*>(b_rows + int64_t(jb) * kHeadDim + kScoreHalf * half + 4 * piece);
    }
  };
  fetch(0);
  for (int half = 0; half < kSlices; ++half) {
    if (half) __syncthreads();                      // everyone is done with the previous slice
#pragma unroll
    for (int x = 0; x < kLoads; ++x) {
      const int idx = tid + 256 * x;
      const int row = idx / kPieces, piece = idx % kPieces;
      *reinterpret_cast<f32x4*>(&a_lds[row * kScoreRow + 4 * piece]) = va[x];
      *reinterpret_cast<f32x4*>(&b_lds[row * kScoreRow + 4 * piece]) = vb[x];
    }
    __syncthreads();
    if (half + 1 < kSlices) fetch(half + 1);
    if (active) {
#pragma unroll
      for (int c = 0; c < kScoreHalf / 8; ++c) {
        f32x4 av[2], bv[2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          av[x] = *reinterpret_cast<const f32x4*>(&a_lds[(64 * wi + 32 * x + n) * kScoreRow + 8 * c + 4 * hi]);
          bv[x] = *reinterpret_cast<const f32x4*>(&b_lds[(64 * wj + 32 * x + n) * kScoreRow + 8 * c + 4 * hi]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int y = 0; y < 2; ++y)
              acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[x][u], bv[y][u], acc[x][y], 0, 0, 0);
      }
    }
  }
  if (!active) return;
  float* out = scores + meta.score_off[s] + int64_t(h) * nb * nb;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int j = j0 + 32 * y + n;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = i0 + 32 * x + 8 * (r >> 2) + 4 * hi + (r & 3);
        if (i < nb && j <= i) out[int64_t(i) * nb + j] = acc[x][y][r] * scale;
      }
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
  const int tiles = (g.max_nb + 127) / 128;
  hipLaunchKernelGGL(score_kernel, dim3(tiles * (tiles + 1) / 2, 1, m.n_seq * m.n_q_heads), dim3(256), 0, stream, m,
                     qbar, kbar, scores, int(g.total_blocks), g.scale);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
