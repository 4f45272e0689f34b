// Block importance: mean-pool query/key blocks (HBM-bound streaming reduction), then
// pooled logits for the causal lower triangle (a small contraction, fp32 values carried
// as three bf16 planes so that it runs on the bf16 matrix pipe).
#include "attn_common.h"

namespace shplb {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

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
// keeps fp32 sums; partial sums meet in LDS in a fixed order (deterministic).  The
// fp32 mean v leaves as three bf16 planes v1 = bf16(v), v2 = bf16(v - v1), v3 = bf16(v - v1 - v2)
// (round to nearest even; the differences are exact in fp32), each plane [heads][blocks][128].
// blockIdx.x enumerates first the Q tiles, then the K tiles.
// Two workgroups per compute unit with 16 loads of 16 bytes in flight per lane: fewer, longer
// streams suit the memory better than full occupancy with 8 in flight (213 against 224 us at
// 128K tokens of a 32/8-head layer).
__global__ __launch_bounds__(kPoolThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void pool_kernel(
    SeqMeta meta, Strides st, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    uint16_t* __restrict__ q_planes, uint16_t* __restrict__ k_planes, int q_chunks, int k_chunks,
    int total_blocks) {
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
  uint16_t* dst = is_q ? q_planes : k_planes;
  const int64_t plane = int64_t(n_heads) * total_blocks * kHeadDim;

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
    constexpr int U = 16;             // loads in flight per lane
    for (; t + (U - 1) * kPoolWaves < t1; t += U * kPoolWaves) {
      u32x4 w[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + int64_t(t + u * kPoolWaves) * stride_t));
#pragma unroll
      for (int u = 0; u < U; ++u) add_bf16x8(acc, w[u]);
    }
    for (; t < t1; t += kPoolWaves) {
      const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + int64_t(t) * stride_t));
      add_bf16x8(acc, w);
    }
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) part[wave][lane * 8 + c] = acc[c];
  __syncthreads();
  {
    const int x = 2 * threadIdx.x;                  // two neighbouring dims per thread
    const int ee = chunk * kPoolElems + x;
    const int hh = ee >> 7, dd = ee & 127;
    if (hh < n_heads) {
      float v0 = (((part[0][x] + part[1][x]) + part[2][x]) + part[3][x]) / float(cnt);
      float v1 = (((part[0][x + 1] + part[1][x + 1]) + part[2][x + 1]) + part[3][x + 1]) / float(cnt);
      if (is_q) {
        // query means stay fp32: the scoring kernel loads each row into registers anyway and splits it
        // there (two thirds of the bytes of three planes, on a buffer that is written once and read 2.5 times)
        float* qm = reinterpret_cast<float*>(q_planes) + (int64_t(hh) * total_blocks + gblk) * kHeadDim + dd;
        *reinterpret_cast<float2*>(qm) = float2{v0, v1};
        return;
      }
      uint16_t* at = dst + (int64_t(hh) * total_blocks + gblk) * kHeadDim + dd;
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) {
        const __bf16 b0 = (__bf16)v0, b1 = (__bf16)v1;
        *reinterpret_cast<uint32_t*>(at + pl * plane) =
            uint32_t(__builtin_bit_cast(uint16_t, b0)) | uint32_t(__builtin_bit_cast(uint16_t, b1)) << 16;
        v0 -= float(b0);
        v1 -= float(b1);
      }
    }
  }
}

// scores[s][h][i][j] = (qbar[h][i] . kbar[h/G][j]) * scale for j <= i.
//
// fp32 products on the bf16 matrix pipe.  The pooling kernel stores every pooled value v as
// three bf16 planes v = v1 + v2 + v3 (v1 = bf16(v), v2 = bf16(v - v1), v3 = bf16(v - v1 - v2):
// all 24 mantissa bits), and a product is taken as q1k1 + q1k2 + q2k1 + q2k2 + q1k3 + q3k1;
// the dropped cross terms are below 2^-24 of the product, what an fp32 multiply rounds away
// anyway.  Six v_mfma_f32_32x32x16_bf16 do the work of eight v_mfma_f32_32x32x2_f32 in
// 3/8 of the time.
//
// One workgroup = 128 query-block rows (32 per wave) of one (sequence, head) x a chunk of
// key-block rows, streamed in tiles of 32 through a double-buffered LDS stage; three
// workgroups share a compute unit and hide each other's copy latency.  The Q planes of a
// wave's rows stay in registers as MFMA B-operands; a K tile is 3 planes x 32 rows of 256
// bytes, copied global->LDS directly and laid out like the K tiles of the attention kernels
// (chunk c of row r at slot c ^ swz(r)).  Lane (n, hi) ends up with row i = n of the 32x32
// output tile and four runs of four consecutive j: 16-byte stores.  Two accumulators take
// the six products in turn (no MFMA waits for the one before it) and are added at the end;
// the order of additions is fixed.
constexpr int kScoreTile = 128;                       // query-block rows per workgroup
constexpr int kScoreJ = 32;                           // key-block rows per LDS stage
constexpr int kPlanes = 3;
constexpr int kScoreStageBytes = kPlanes * kScoreJ * kRowBytes;   // 24 KB
// chunks (of `chunk` key-block rows) that hold some j <= i for the rows of tile row tr
__host__ __device__ constexpr int score_chunks_of_row(int tr, int chunk) {
  return (tr * kScoreTile + kScoreTile - 1) / chunk + 1;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void score_kernel(
    SeqMeta meta, const uint16_t* __restrict__ q_planes, const uint16_t* __restrict__ k_planes,
    float* __restrict__ scores, int total_blocks, int chunk, float scale) {
  __shared__ __attribute__((aligned(1024))) char k_lds[2][kScoreStageBytes];
  const int sh = blockIdx.z;
  const int s = sh / meta.n_q_heads, h = sh - s * meta.n_q_heads;
  const int nb = meta.blk_begin[s + 1] - meta.blk_begin[s];
  // blockIdx.x enumerates (128-row tile of query blocks, chunk of key blocks) pairs of the
  // lower triangle, tile row by tile row.  Consecutive workgroup ids go to different XCDs,
  // so every die gets the same share of live work (a square grid would hand die x the whole
  // chunk column x, most of which lies above the diagonal for large x).
  int tr = 0, rest = int(blockIdx.x);
  while (rest >= score_chunks_of_row(tr, chunk)) rest -= score_chunks_of_row(tr++, chunk);
  const int ti = tr * kScoreTile, tj = rest * chunk;
  if (ti >= nb) return;                             // shorter sequence of a varlen batch
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hi = lane >> 5;
  const int g = kv_head_of(meta, h);
  const int i_first = ti + 32 * wave;               // this wave's rows
  const int i_last = min(ti + kScoreTile, nb) - 1;  // last row of the workgroup
  if (tj > i_last) return;                          // chunk entirely right of a short sequence's last row (before any copy is issued)
  const int n_jt = (min(tj + chunk, i_last + 1) - tj + kScoreJ - 1) / kScoreJ;   // 32-row K tiles with some j <= i
  const int64_t k_plane = int64_t(meta.n_kv_heads) * total_blocks * kHeadDim;
  const char* k_rows = reinterpret_cast<const char*>(k_planes + (int64_t(g) * total_blocks + meta.blk_begin[s]) * kHeadDim);

  // copies: round rd of a tile fills LDS rows 16rd .. 16rd+15 = plane rd/2, tile rows 16(rd&1)..;
  // this lane's row inside the tile and its slot are the same in every round of one parity
  const int cp_jl = 4 * wave + (lane >> 4);
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_offset_of(&k_lds[0][0]) + 4 * wave * kRowBytes);
  auto issue_tile = [&](int jt, int stage) __attribute__((always_inline)) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int jl = 16 * half + cp_jl;
      const int j = min(tj + kScoreJ * jt + jl, nb - 1);          // rows past the end repeat the last one (never stored)
      const uint32_t off = uint32_t(j) * kRowBytes + (((lane & 15) ^ swz(jl)) << 4);
#pragma unroll
      for (int pl = 0; pl < kPlanes; ++pl)
        copy_g2l_16(k_rows + pl * k_plane * 2, off, lds0 + stage * kScoreStageBytes + (2 * pl + half) * 16 * kRowBytes);
    }
  };
  issue_tile(0, 0);

  // Q planes of row i_first + n: B operands, lane (n, hi) holds dims 16ks + 8hi .. +7.  The means arrive
  // as fp32 and are split here into the three bf16 planes (v1 = bf16(v), v2 = bf16(v - v1),
  // v3 = bf16(v - v1 - v2); the differences are exact), as the pooling kernel does for the keys.
  bf16x8 qf[kPlanes][8];
  {
    const int i = min(i_first + n, nb - 1);
    const float* src = reinterpret_cast<const float*>(q_planes) +
                       (int64_t(h) * total_blocks + meta.blk_begin[s] + i) * kHeadDim + 8 * hi;
    f32x4 raw[8][2];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      raw[ks][0] = *reinterpret_cast<const f32x4*>(src + 16 * ks);
      raw[ks][1] = *reinterpret_cast<const f32x4*>(src + 16 * ks + 4);
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float v = raw[ks][c >> 2][c & 3];
#pragma unroll
        for (int pl = 0; pl < kPlanes; ++pl) {
          const __bf16 b = (__bf16)v;
          qf[pl][ks][c] = b;
          v -= float(b);
        }
      }
  }
  typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;
  const uint32_t k_rd0 = lds_offset_of(&k_lds[0][0]) + uint32_t(n * kRowBytes + ((hi ^ swz(n)) << 4));
  auto read_k = [&](int stage, int pl, int ks) __attribute__((always_inline)) {
    return *reinterpret_cast<lds_bf16x8*>((k_rd0 ^ uint32_t(ks << 5)) + uint32_t(stage * kScoreStageBytes + pl * kScoreJ * kRowBytes));
  };
  float* out = scores + meta.score_off[s] + int64_t(h) * nb * nb;

  // Lane (n, hi) holds row i = i_first + n of a finished tile, columns j0 + 8(r/4) + 4hi + (r%4):
  // four runs of four.
  auto store_tile = [&](const f32x16& v16, int j0) __attribute__((always_inline)) {
    const int i = i_first + n;
    if (i >= nb) return;
    float* row = out + int64_t(i) * nb + j0 + 4 * hi;
    const bool aligned = (reinterpret_cast<uintptr_t>(row) & 15) == 0;   // odd block counts shift rows
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int j = j0 + 8 * rq + 4 * hi;
      const f32x4 v = {v16[4 * rq], v16[4 * rq + 1], v16[4 * rq + 2], v16[4 * rq + 3]};
      if (j + 3 <= i && aligned) {
        *reinterpret_cast<f32x4*>(row + 8 * rq) = v;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (j + c <= i) row[8 * rq + c] = v[c];
      }
    }
  };

  // A finished tile is written out one iteration later, behind the barrier: the wait at
  // the top of an iteration covers every memory operation of the wave (a wave's loads and
  // stores need not complete in order, so a count would not do), and stores issued just
  // before it would make each iteration pay their full latency.
  f32x16 pend;
  int pend_j0 = -1;
  for (int jt = 0; jt < n_jt; ++jt) {
    const int stage = jt & 1;
    wait_vmem_all();                                // own copies of tile jt have landed
    __syncthreads();                                // everyone's have; the other stage is free
    if (jt + 1 < n_jt) issue_tile(jt + 1, stage ^ 1);
    if (pend_j0 >= 0) {
      store_tile(pend, pend_j0);
      pend_j0 = -1;
    }
    const int j0 = tj + kScoreJ * jt;
    if (j0 > i_first + 31) continue;                // tile entirely above this wave's rows (uniform per wave)
    f32x16 acc_a, acc_b;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_a[r] = acc_b[r] = 0.0f;
    bf16x8 kf[2][kPlanes];
#pragma unroll
    for (int pl = 0; pl < kPlanes; ++pl) kf[0][pl] = read_k(stage, pl, 0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const int cur = ks & 1;
      if (ks + 1 < 8) {
#pragma unroll
        for (int pl = 0; pl < kPlanes; ++pl) kf[cur ^ 1][pl] = read_k(stage, pl, ks + 1);
      }
      acc_a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][0], qf[0][ks], acc_a, 0, 0, 0);
      acc_b = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][1], qf[0][ks], acc_b, 0, 0, 0);
      acc_a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][0], qf[1][ks], acc_a, 0, 0, 0);
      acc_b = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][1], qf[1][ks], acc_b, 0, 0, 0);
      acc_a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][2], qf[0][ks], acc_a, 0, 0, 0);
      acc_b = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][0], qf[2][ks], acc_b, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) pend[r] = (acc_a[r] + acc_b[r]) * scale;
    pend_j0 = j0;
  }
  if (pend_j0 >= 0) store_tile(pend, pend_j0);
}

}  // namespace

int32_t launch_pool_scores(const Geometry& g, const void* q, const void* k, float* scores,
                           uint16_t* q_planes, uint16_t* k_planes, int n_compute_units, hipStream_t stream) {
  const SeqMeta& m = g.meta;
  const int q_chunks = (m.n_q_heads * kHeadDim + kPoolElems - 1) / kPoolElems;
  const int k_chunks = (m.n_kv_heads * kHeadDim + kPoolElems - 1) / kPoolElems;
  const int64_t n_wg = g.total_blocks * (q_chunks + k_chunks);
  if (n_wg > 0x7fffffff) return SHPLB_E_UNSUPPORTED;
  hipLaunchKernelGGL(pool_kernel, dim3(uint32_t(n_wg)), dim3(kPoolThreads), 0, stream, m, g.st,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), q_planes, k_planes,
                     q_chunks, k_chunks, int(g.total_blocks));
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  // Key-block rows per workgroup: the shortest chunk with which the whole launch is resident at
  // once (three workgroups per compute unit); more, shorter workgroups would run in rounds,
  // fewer, longer ones would leave compute units idle.
  const int tiles = (g.max_nb + kScoreTile - 1) / kScoreTile;
  const int64_t resident = int64_t(n_compute_units) * 3;
  int chunk = 64, n_pairs = 0;
  for (;; chunk *= 2) {
    n_pairs = 0;
    for (int tr = 0; tr < tiles; ++tr) n_pairs += score_chunks_of_row(tr, chunk);
    if (int64_t(n_pairs) * m.n_seq * m.n_q_heads <= resident || chunk >= tiles * kScoreTile) break;
  }
  hipLaunchKernelGGL(score_kernel, dim3(n_pairs, 1, m.n_seq * m.n_q_heads), dim3(256), 0, stream, m,
                     q_planes, k_planes, scores, int(g.total_blocks), chunk, g.scale);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
