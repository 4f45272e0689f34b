// Block-sparse causal attention over per-row selected key blocks (gfx950).
//
// Work item = one (sequence, head, query block) row of the selection.  Persistent
// workgroups draw items from a cost-descending list through one atomic ticket.
//
// Tiling (wave64, v_mfma_f32_32x32x16_bf16):
//   * each wave owns 32*NT query rows and keeps Q as MFMA B-operands in registers;
//     with NT = 1 a 128-row query block is 4 waves and two workgroups share a compute
//     unit, so every SIMD holds two waves of different workgroups: one wave's softmax
//     VALU work overlaps the other's MFMAs;
//   * keys are streamed in sub-tiles of 64 through a double-buffered LDS stage; K and V
//     are both stored row-major ([key][dim]); K is read as an MFMA A-operand with
//     16-byte LDS reads, V through the LDS transpose read (ds_read_b64_tr_b16), which
//     hands each lane four keys of one dim;
//   * the first contraction is S^T = K Q^T, so a lane holds one query column: the
//     softmax max/sum are in-lane plus one exchange with lane^32, and the
//     probabilities feed the second contraction O^T += V^T P^T straight from
//     registers (the key order inside a 16-key MFMA step is permuted identically
//     on both operands, which a sum over keys does not see);
//   * the running maximum is only raised (and O, l rescaled) when some row's tile
//     maximum exceeds it by more than 2^8; in between, probabilities are taken
//     relative to the stale maximum, which the final division by l cancels exactly.
#include "shplb_internal.h"

namespace shplb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kKeysPerTile = 64;
constexpr int kKRow = 136;   // halfs per K row in LDS (128 + 8 pad -> 272 B, conflict-free b128 reads)
constexpr int kVRow = 144;   // halfs per V row in LDS (128 + 16 pad -> 288 B, conflict-free transpose reads)
constexpr int kKTile = kKeysPerTile * kKRow;
constexpr int kVTile = kKeysPerTile * kVRow;
constexpr float kRescaleSlack = 8.0f;   // log2 units a row maximum may grow before O, l are rescaled

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, v);
}

typedef short s16x4 __attribute__((ext_vector_type(4)));

// LDS transpose read: inside every group of 16 lanes, lane L receives element L%4 of
// the four 8-byte pieces addressed by lanes L/4, L/4+4, L/4+8, L/4+12.
__device__ __forceinline__ s16x4 lds_read_tr16(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(p));
}

template <int BQ, int NT>
struct AttnCfg {
  static constexpr int kWaves = BQ / (32 * NT);
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kWavesPerSimd = NT == 1 ? 2 : 1;
  static constexpr int kKChunks = kKeysPerTile * 16 / kThreads;     // 16-byte pieces of K per thread
};

template <int BQ, int NT>
__global__ __launch_bounds__(64 * (BQ / (32 * NT)))
__attribute__((amdgpu_waves_per_eu(NT == 1 ? 2 : 1, NT == 1 ? 2 : 1)))
void attn_kernel(SeqMeta meta, Strides st, const uint16_t* __restrict__ q,
                 const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                 const int64_t* __restrict__ sel_ptr, const int32_t* __restrict__ sel_idx,
                 uint16_t* __restrict__ out, float* __restrict__ lse, shplb_wg_stats* __restrict__ stats,
                 const int32_t* __restrict__ order, uint32_t* __restrict__ ticket, int32_t rows,
                 int64_t total_tokens, float scale_log2) {
  using Cfg = AttnCfg<BQ, NT>;
  constexpr int kThreads = Cfg::kThreads;
  constexpr int SUB = BQ / kKeysPerTile;   // 64-key sub-tiles per key block
  constexpr int QW = 32 * NT;              // queries per wave
  constexpr int KC = Cfg::kKChunks;

  __shared__ __attribute__((aligned(16))) uint16_t k_lds[2][kKTile];
  __shared__ __attribute__((aligned(16))) uint16_t v_lds[2][kVTile];
  __shared__ int32_t s_item;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int group = meta.n_q_heads / meta.n_kv_heads;

  uint32_t my_items = 0, my_cost = 0;
  uint64_t t_first = 0, t_last = 0;

  for (;;) {
    if (tid == 0) s_item = int32_t(atomicAdd(ticket, 1u));
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(s_item);   // uniform: keep the item's geometry in SGPRs
    __syncthreads();
    if (item >= rows) break;
    const int row = order[item];
    int s, h, i, nb;
    decode_row(meta, row, s, h, i, nb);
    const int g = h / group;
    const int seq_begin = meta.tok_begin[s], seq_end = meta.tok_begin[s + 1];
    const int64_t sel_begin = sel_ptr[row];
    const int n_sel = int(sel_ptr[row + 1] - sel_begin);
    const int n_tiles = n_sel * SUB;
    if (n_sel <= 0) continue;          // malformed row: nothing to attend to
    if (my_items == 0) t_first = wall_clock64();
    my_items += 1;
    my_cost += uint32_t(n_sel);

    // ---- Q fragments: B operand of S^T = K Q^T, lane (n, hi) holds dims 16ks+8hi.. of its query
    bf16x8 qf[NT][8];
    int q_tok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      q_tok[nt] = seq_begin + i * BQ + wave * QW + 32 * nt + n;
      const int tok = min(q_tok[nt], seq_end - 1);
      const uint16_t* src = q + int64_t(tok) * st.q_t + int64_t(h) * st.q_h + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) qf[nt][ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
    }

    f32x16 acc_o[4][NT];
    float m_ref[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      m_ref[nt] = -INFINITY;
      l_run[nt] = 0.0f;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][nt][r] = 0.0f;
    }

    const char* k_head = reinterpret_cast<const char*>(k + int64_t(g) * st.kv_h);
    const char* v_head = reinterpret_cast<const char*>(v + int64_t(g) * st.kv_h);
    const int64_t row_bytes = st.kv_t * 2;
    // per-thread byte offsets inside a 64-key tile (constant over tiles); the tile's base
    // and the per-chunk row steps are wave-uniform and stay in scalar registers
    const uint32_t k_off = uint32_t((tid >> 4) * row_bytes + (tid & 15) * 16);
    u32x4 k_regs[KC], v_regs[KC];

    auto load_tile = [&](int it) {
      const int p = it / SUB, sub = it - p * SUB;
      const int j = min(max(sel_idx[sel_begin + p], 0), nb - 1);
      const int key_base = seq_begin + j * BQ + kKeysPerTile * sub;
      const int valid = seq_end - key_base;            // keys of this tile inside the sequence
      const char* kt = k_head + int64_t(key_base) * row_bytes;
      const char* vt = v_head + int64_t(key_base) * row_bytes;
      if (valid >= kKeysPerTile) {
#pragma unroll
        for (int c = 0; c < KC; ++c)
          k_regs[c] = *reinterpret_cast<const u32x4*>(kt + int64_t(c * (kThreads / 16)) * row_bytes + k_off);
#pragma unroll
        for (int c = 0; c < KC; ++c)
          v_regs[c] = *reinterpret_cast<const u32x4*>(vt + int64_t(c * (kThreads / 16)) * row_bytes + k_off);
      } else {                                          // ragged last block: clamp to the last valid key
#pragma unroll
        for (int c = 0; c < KC; ++c) {
          const int tok = min(key_base + (tid >> 4) + c * (kThreads / 16), seq_end - 1);
          k_regs[c] = *reinterpret_cast<const u32x4*>(k_head + int64_t(tok) * row_bytes + (tid & 15) * 16);
          v_regs[c] = *reinterpret_cast<const u32x4*>(v_head + int64_t(tok) * row_bytes + (tid & 15) * 16);
        }
      }
    };

    auto store_tile = [&](int buf) {
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        const int x = tid + kThreads * c;
        *reinterpret_cast<u32x4*>(&k_lds[buf][(x >> 4) * kKRow + (x & 15) * 8]) = k_regs[c];
        *reinterpret_cast<u32x4*>(&v_lds[buf][(x >> 4) * kVRow + (x & 15) * 8]) = v_regs[c];
      }
    };

    // transpose-read addressing of V: lane = 16*grp + 4*e + a supplies the piece
    // (key 4*hi + e, dims 16*(grp&1) + 4a ..) and receives keys 4*hi + 0..3 of dim
    // 16*(grp&1) + (lane&15) = lane&31, i.e. the A-operand of its own MFMA row.
    const int v_rd = (4 * hi + ((lane >> 2) & 3)) * kVRow + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    load_tile(0);
    store_tile(0);
    if (n_tiles > 1) load_tile(1);
    __syncthreads();

    for (int it = 0; it < n_tiles; ++it) {
      const int buf = it & 1;
      // stage the next tile (its buffer was last read one iteration ago, before the barrier)
      if (it + 1 < n_tiles) store_tile(buf ^ 1);
      if (it + 2 < n_tiles) load_tile(it + 2);

      const int p = it / SUB, sub = it - p * SUB;
      const bool diag = sel_idx[sel_begin + p] == i;
      // a diagonal sub-tile entirely above this wave's queries contributes nothing
      const bool skip = diag && kKeysPerTile * sub > wave * QW + QW - 1;
      if (!skip) {
        const uint16_t* kt = k_lds[buf];
        const uint16_t* vt = v_lds[buf];

        // ---- S^T = K Q^T : [64 keys] x [QW queries]
        f32x16 sc[2][NT];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[mt][nt][r] = 0.0f;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(&kt[(32 * mt + n) * kKRow + 16 * ks + 8 * hi]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              sc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nt][ks], sc[mt][nt], 0, 0, 0);
          }
        }

        // ---- online softmax (log2 domain), one query column per lane
        bf16x8 pf[NT][4];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          if (diag) {
            const int q_in = wave * QW + 32 * nt + n;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int key_in = kKeysPerTile * sub + 32 * mt + 8 * (r >> 2) + 4 * hi + (r & 3);
                if (key_in > q_in) sc[mt][nt][r] = -INFINITY;
              }
          }
          float mx = fmaxf(sc[0][nt][0], sc[1][nt][0]);
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(sc[0][nt][r], sc[1][nt][r]));
          mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;
          if (__any(mx > m_ref[nt] + kRescaleSlack)) {
            const float m_new = fmaxf(m_ref[nt], mx);
            const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref[nt] - m_new);
            m_ref[nt] = m_new;
            l_run[nt] *= alpha;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
              for (int r = 0; r < 16; ++r) acc_o[dt][nt][r] *= alpha;
          }
          const float m_use = m_ref[nt] == -INFINITY ? 0.0f : m_ref[nt];
          float rs = 0.0f;
          uint32_t pk[2][8];
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
              const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[mt][nt][r], scale_log2, -m_use));
              const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[mt][nt][r + 1], scale_log2, -m_use));
              rs += p0 + p1;
              pk[mt][r >> 1] = pack_bf16(p0, p1);
            }
          l_run[nt] += rs;
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const u32x4 w = {pk[gq >> 1][4 * (gq & 1)], pk[gq >> 1][4 * (gq & 1) + 1],
                             pk[gq >> 1][4 * (gq & 1) + 2], pk[gq >> 1][4 * (gq & 1) + 3]};
            pf[nt][gq] = __builtin_bit_cast(bf16x8, w);
          }
        }

        // ---- O^T += V^T P^T : [128 dims] x [QW queries], 16 keys per MFMA step
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            // keys 16gq + 4hi + {0..3} and 16gq + 8 + 4hi + {0..3} of dim 32dt + n
            const s16x4 lo = lds_read_tr16(&vt[v_rd + (16 * gq) * kVRow + 32 * dt]);
            const s16x4 hi4 = lds_read_tr16(&vt[v_rd + (16 * gq + 8) * kVRow + 32 * dt]);
            const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc_o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[nt][gq], acc_o[dt][nt], 0, 0, 0);
          }
        }
      }
      __syncthreads();
    }

    // ---- normalise and store: lane holds, for its query, dims 32dt + 8(r/4) + 4hi + (r%4)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const float l_tot = l_run[nt] + __shfl_xor(l_run[nt], 32);
      if (q_tok[nt] < seq_end) {
        const float inv = 1.0f / l_tot;
        uint16_t* dst = out + int64_t(q_tok[nt]) * st.q_t + int64_t(h) * st.q_h + 4 * hi;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            u32x2 w;
            w.x = pack_bf16(acc_o[dt][nt][4 * rq] * inv, acc_o[dt][nt][4 * rq + 1] * inv);
            w.y = pack_bf16(acc_o[dt][nt][4 * rq + 2] * inv, acc_o[dt][nt][4 * rq + 3] * inv);
            *reinterpret_cast<u32x2*>(dst + 32 * dt + 8 * rq) = w;
          }
        if (lse != nullptr && hi == 0)
          lse[int64_t(h) * total_tokens + q_tok[nt]] =
              (m_ref[nt] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
      }
    }
    t_last = wall_clock64();
  }

  if (stats != nullptr && tid == 0) {
    shplb_wg_stats rec;
    rec.xcc_id = __builtin_amdgcn_s_getreg((4 - 1) << 11 | 0 << 6 | 20) & 0xf;       // XCC_ID[3:0]
    rec.cu_id = (__builtin_amdgcn_s_getreg((16 - 1) << 11 | 0 << 6 | 4) >> 8) & 0xff; // HW_ID[15:8]
    rec.n_items = my_items;
    rec.cost_blocks = my_cost;
    rec.t_first = t_first;
    rec.t_last = t_last;
    stats[blockIdx.x] = rec;
  }
}

template <int BQ, int NT>
void launch_one(const Geometry& g, const void* q, const void* k, const void* v, const int64_t* sel_ptr,
                const int32_t* sel_idx, void* out, float* lse, shplb_wg_stats* stats,
                const int32_t* order, uint32_t* ticket, int32_t n_wg, hipStream_t stream) {
  const float scale_log2 = g.scale * 1.4426950408889634f;
  hipLaunchKernelGGL((attn_kernel<BQ, NT>), dim3(n_wg), dim3(AttnCfg<BQ, NT>::kThreads), 0, stream, g.meta,
                     g.st, static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                     static_cast<const uint16_t*>(v), sel_ptr, sel_idx, static_cast<uint16_t*>(out), lse,
                     stats, order, ticket, int32_t(g.rows), g.total_tokens, scale_log2);
}

}  // namespace

int32_t launch_attention(const Geometry& g, const void* q, const void* k, const void* v,
                         const int64_t* sel_ptr, const int32_t* sel_idx, void* out, float* lse,
                         shplb_wg_stats* stats, const int32_t* order, uint32_t* ticket,
                         int32_t n_wg, hipStream_t stream) {
  if (g.meta.block == 128)
    launch_one<128, 1>(g, q, k, v, sel_ptr, sel_idx, out, lse, stats, order, ticket, n_wg, stream);
  else
    launch_one<64, 1>(g, q, k, v, sel_ptr, sel_idx, out, lse, stats, order, ticket, n_wg, stream);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
