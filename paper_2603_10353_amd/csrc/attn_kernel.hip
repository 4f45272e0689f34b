// Block-sparse causal attention over per-row selected key blocks (gfx950).
//
// Work item = one (sequence, head, query block) row of the selection.  Persistent
// workgroups draw items from a cost-descending list through one atomic ticket.
//
// Tiling (wave64, v_mfma_f32_32x32x16_bf16):
//   * a wave owns 32 query rows and keeps Q as MFMA B-operands in registers; a
//     128-row query block is 4 waves and two workgroups share a compute unit, so every
//     SIMD holds two waves of different workgroups: one wave's softmax VALU work
//     overlaps the other's MFMAs;
//   * keys are streamed in sub-tiles of 64.  K and V rows go from global memory
//     straight into a double-buffered LDS stage (global_load_lds_dwordx4, no staging
//     registers, no LDS store instructions).  Rows are 256 bytes, unpadded; the
//     16-byte chunk c of row r sits at chunk slot c ^ swz(r), which keeps both the K
//     operand reads and the V transpose reads free of bank conflicts;
//   * the first contraction is S^T = K Q^T (A = K from LDS by 16-byte reads), so a
//     lane holds one query column: the softmax max/sum are in-lane plus one exchange
//     with lane^32, and the probabilities feed the second contraction
//     O^T += V^T P^T straight from registers (the key order inside a 16-key MFMA step
//     is permuted identically on both operands, which a sum over keys does not see);
//     V^T operands come from the LDS transpose read (ds_read_b64_tr_b16);
//   * all LDS operand reads of a phase are issued ahead of its MFMAs, so the MFMAs
//     run back to back;
//   * the running maximum is only raised (and O, l rescaled) when some row's tile
//     maximum exceeds it by more than 2^8; in between, probabilities are taken
//     relative to the stale maximum, which the final division by l cancels exactly.
#include "attn_common.h"

namespace shplb {

namespace {

template <int BQ>
__global__ __launch_bounds__(2 * BQ) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_kernel(SeqMeta meta, Strides st, const uint16_t* __restrict__ q,
                 const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                 const int64_t* __restrict__ sel_ptr, const int32_t* __restrict__ sel_idx,
                 uint16_t* __restrict__ out, float* __restrict__ lse, shplb_wg_stats* __restrict__ stats,
                 WorkQueues wq, SplitBuffers sb, int64_t total_tokens, float scale_log2) {
  constexpr int kWaves = BQ / 32;
  constexpr int SUB = BQ / kKeysPerTile;            // 64-key sub-tiles per key block
  constexpr int kRoundRows = 4 * kWaves;            // rows one round of copies moves (4 per wave)
  constexpr int kRounds = kKeysPerTile / kRoundRows;

  __shared__ __attribute__((aligned(1024))) char k_lds[2][kTileBytes];
  __shared__ __attribute__((aligned(1024))) char v_lds[2][kTileBytes];
  __shared__ int32_t s_item;
  __shared__ int32_t s_flag;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hi = lane >> 5;

  // ---- per-lane constants
  // global->LDS copies: lane (r4 = lane>>4, slot = lane&15) of a wave fills LDS row
  // base + r4, slot `slot`, with the source chunk slot ^ swz(row).
  const int cp_row = 4 * wave + (lane >> 4);
  // K operand reads: lane (n, hi) reads row 32mt + n, chunk 2ks + hi.
  const int k_rd0 = n * kRowBytes + ((hi ^ swz(n)) << 4);                 // ks = 0; other ks: ^ (ks << 5)
  // V transpose reads: lane = 16*grp + 4e + a supplies the piece (key 16gq + 8half + 4hi + e,
  // dims 32dt + 16(grp&1) + 4a ..) and receives keys 4hi+0..3 (+8half, +16gq) of dim 32dt + n.
  const int tr_e = (lane >> 2) & 3, tr_a = lane & 3, tr_mh = (lane >> 4) & 1;
  int v_rd0[2];                                                            // dt = 0; other dt: ^ (dt << 6)
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int r = 8 * half + 4 * hi + tr_e;
    v_rd0[half] = r * kRowBytes + (((2 * tr_mh + (tr_a >> 1)) ^ swz(r)) << 4) + 8 * (tr_a & 1);
  }

  // LDS byte offsets of this wave's 1 KB slice inside round 0 of stage 0
  const uint32_t k_stage0 = __builtin_amdgcn_readfirstlane(lds_offset_of(&k_lds[0][0]) + 4 * wave * kRowBytes);
  const uint32_t v_stage0 = __builtin_amdgcn_readfirstlane(lds_offset_of(&v_lds[0][0]) + 4 * wave * kRowBytes);

  uint32_t my_items = 0, my_cost = 0;
  uint64_t t_first = 0, t_last = 0;
  const int home = my_xcd();
  int empty_mask = 0;                    // queues this workgroup has found empty (thread 0 only)

  for (;;) {
    if (tid == 0) s_item = next_item(wq, home, empty_mask);
    __syncthreads();
    const int pos = __builtin_amdgcn_readfirstlane(s_item);   // uniform: keep the item's geometry in SGPRs
    __syncthreads();
    if (pos < 0) break;
    // the item: a row, or a piece of one (then it covers part of the row's selection and
    // leaves a partial result in a slot instead of the output)
    const ItemRec* item = wq.items + pos;
    const int row = __builtin_amdgcn_readfirstlane(item->row);
    const int n_sel = __builtin_amdgcn_readfirstlane(item->n_sel);
    const int64_t sel_begin = item->sel_begin;
    const int slot = __builtin_amdgcn_readfirstlane(item->slot);
    if (row < 0 || row >= meta.blk_begin[meta.n_seq] * meta.n_q_heads || slot >= sb.slot_capacity) continue;
    int s, h, i, nb;
    decode_row(meta, row, s, h, i, nb);
    const int g = kv_head_of(meta, h);
    const int seq_begin = meta.tok_begin[s], seq_end = meta.tok_begin[s + 1];
    const int n_tiles = n_sel * SUB;
    if (n_sel <= 0) continue;          // malformed row: nothing to attend to
    if (my_items == 0) t_first = wall_clock64();
    my_items += 1;
    my_cost += uint32_t(n_sel);

    const char* k_head = reinterpret_cast<const char*>(k + int64_t(g) * st.kv_h);
    const char* v_head = reinterpret_cast<const char*>(v + int64_t(g) * st.kv_h);
    const int64_t row_bytes = st.kv_t * 2;

    // Copy tile `it` (64 keys of K and of V) from global memory into LDS stage `buf`.
    auto issue_tile = [&](int it, int buf) {
      const int p = it / SUB, sub = it - p * SUB;
      const int j = min(max(sel_idx[sel_begin + p], 0), nb - 1);
      // A sub-tile that starts past the end of a ragged last block is moved back onto the
      // last token: every row offset below must stay non-negative (it is added unsigned).
      const int key_base = min(seq_begin + j * BQ + kKeysPerTile * sub, seq_end - 1);
      const int last = seq_end - 1 - key_base;                 // last valid row of the tile (0 .. or >= 63)
      const char* k_tile = k_head + int64_t(key_base) * row_bytes;
      const char* v_tile = v_head + int64_t(key_base) * row_bytes;
      const uint32_t k_dst = k_stage0 + buf * kTileBytes, v_dst = v_stage0 + buf * kTileBytes;
#pragma unroll
      for (int rd = 0; rd < kRounds; ++rd) {
        const int r = rd * kRoundRows + cp_row;                // LDS row this lane fills
        const int src_col = ((lane & 15) ^ swz(r)) << 4;
        // rows past the end of the sequence (ragged last block) re-read the last valid key; they are masked
        const uint32_t off = uint32_t(min(r, last)) * uint32_t(row_bytes) + src_col;
        copy_g2l_16(k_tile, off, k_dst + rd * kRoundRows * kRowBytes);
        copy_g2l_16(v_tile, off, v_dst + rd * kRoundRows * kRowBytes);
      }
    };

    issue_tile(0, 0);

    // ---- Q fragments: B operand of S^T = K Q^T, lane (n, hi) holds dims 16ks+8hi.. of its query
    bf16x8 qf[8];
    const int q_tok = seq_begin + i * BQ + wave * 32 + n;
    {
      const int tok = min(q_tok, seq_end - 1);
      const uint16_t* src = q + int64_t(tok) * st.q_t + int64_t(h) * st.q_h + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
    }

    f32x16 acc_o[4];
    float m_ref = -INFINITY, l_run = 0.0f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[dt][r] = 0.0f;

    for (int it = 0; it < n_tiles; ++it) {
      const int buf = it & 1;
      wait_vmem_all();                 // this wave's share of tile `it` has landed in LDS
      __syncthreads();                 // ... and everyone's; everyone is also done reading stage buf^1
      if (it + 1 < n_tiles) issue_tile(it + 1, buf ^ 1);

      const int p = it / SUB, sub = it - p * SUB;
      const bool diag = sel_idx[sel_begin + p] == i;
      // a diagonal sub-tile entirely above this wave's queries contributes nothing
      const bool skip = diag && kKeysPerTile * sub > wave * 32 + 31;
      if (!skip) {
        const char* kt = k_lds[buf];
        const char* vt = v_lds[buf];

        // ---- S^T = K Q^T : [64 keys] x [32 queries]; all 16 K operands fetched up front
        bf16x8 kf[2][8];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            kf[mt][ks] = *reinterpret_cast<const bf16x8*>(kt + (k_rd0 ^ (ks << 5)) + mt * 32 * kRowBytes);
        __builtin_amdgcn_sched_barrier(0);
        f32x16 sc[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) sc[mt][r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
            sc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][ks], qf[ks], sc[mt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);

        // ---- V^T operands for the second contraction, fetched while the softmax runs:
        // keys 16gq + 4hi + {0..3} and 16gq + 8 + 4hi + {0..3} of dim 32dt + n
        s16x4 vf[4][4][2];
#pragma unroll
        for (int gq = 0; gq < 4; ++gq)
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int half = 0; half < 2; ++half)
              vf[gq][dt][half] = lds_read_tr16(vt + (v_rd0[half] ^ (dt << 6)) + gq * 16 * kRowBytes);
        __builtin_amdgcn_sched_barrier(0);

        // ---- online softmax (log2 domain), one query column per lane
        if (diag) {
          const int q_in = wave * 32 + n;
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key_in = kKeysPerTile * sub + 32 * mt + 8 * (r >> 2) + 4 * hi + (r & 3);
              if (key_in > q_in) sc[mt][r] = -INFINITY;
            }
        }
        float mx = fmaxf(sc[0][0], sc[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(sc[0][r], sc[1][r]));
        mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;
        if (__any(mx > m_ref + kRescaleSlack)) {
          const float m_new = fmaxf(m_ref, mx);
          const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);
          m_ref = m_new;
          l_run *= alpha;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[dt][r] *= alpha;
        }
        const float m_use = m_ref == -INFINITY ? 0.0f : m_ref;
        // exponentials first, sums and bf16 packing afterwards: no use sits right behind its exp
        float pr[2][16];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            pr[mt][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[mt][r], scale_log2, -m_use));
        float rs0 = 0.0f, rs1 = 0.0f;
        uint32_t pk[2][8];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            rs0 += pr[mt][r];
            rs1 += pr[mt][r + 1];
            pk[mt][r >> 1] = pack_bf16(pr[mt][r], pr[mt][r + 1]);
          }
        const float rs = rs0 + rs1;
        l_run += rs;
        __builtin_amdgcn_sched_barrier(0);

        // ---- O^T += V^T P^T : [128 dims] x [32 queries], 16 keys per MFMA step
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const u32x4 w = {pk[gq >> 1][4 * (gq & 1)], pk[gq >> 1][4 * (gq & 1) + 1],
                           pk[gq >> 1][4 * (gq & 1) + 2], pk[gq >> 1][4 * (gq & 1) + 3]};
          const bf16x8 pf = __builtin_bit_cast(bf16x8, w);
#pragma unroll
          for (int dt = 0; dt < 4; ++dt) {
            const bf16x8 a = __builtin_bit_cast(
                bf16x8, __builtin_shufflevector(vf[gq][dt][0], vf[gq][dt][1], 0, 1, 2, 3, 4, 5, 6, 7));
            acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, acc_o[dt], 0, 0, 0);
          }
        }
      }
    }

    // ---- normalise and store: lane holds, for its query, dims 32dt + 8(r/4) + 4hi + (r%4)
    {
      const float l_tot = l_run + __shfl_xor(l_run, 32);
      if (slot >= 0) {
        // a piece of a split row: O and l as they stand (relative to 2^m_ref), for finish_piece()
        const int q_in = wave * 32 + n;
        float* part = sb.part_o + int64_t(slot) * kSlotFloatsO;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            float* dst = part + slot_chunk(wave, dt, rq, lane);
            slot_store(dst, acc_o[dt][4 * rq], acc_o[dt][4 * rq + 1]);
            slot_store(dst + 2, acc_o[dt][4 * rq + 2], acc_o[dt][4 * rq + 3]);
          }
        if (hi == 0) {
          float* ml = sb.part_ml + int64_t(slot) * kSlotFloatsML;
          slot_store1(ml + q_in, m_ref);
          slot_store1(ml + 128 + q_in, l_tot);
        }
      } else if (q_tok < seq_end) {
        const float inv = 1.0f / l_tot;
        uint16_t* dst = out + int64_t(q_tok) * st.q_t + int64_t(h) * st.q_h + 4 * hi;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            u32x2 w;
            w.x = pack_bf16(acc_o[dt][4 * rq] * inv, acc_o[dt][4 * rq + 1] * inv);
            w.y = pack_bf16(acc_o[dt][4 * rq + 2] * inv, acc_o[dt][4 * rq + 3] * inv);
            *reinterpret_cast<u32x2*>(dst + 32 * dt + 8 * rq) = w;
          }
        if (lse != nullptr && hi == 0)
          lse[int64_t(h) * total_tokens + q_tok] = (m_ref + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
      }
    }
    if (slot >= 0) {
      const int q0 = seq_begin + i * BQ;
      finish_piece<BQ, 2 * BQ>(sb, item->pieces, item->first_slot, item->split_index,
                               out + int64_t(q0) * st.q_t + int64_t(h) * st.q_h, st.q_t,
                               lse != nullptr ? lse + int64_t(h) * total_tokens + q0 : nullptr,
                               min(BQ, seq_end - q0), &s_flag, reinterpret_cast<float*>(&k_lds[0][0]),
                                 reinterpret_cast<float*>(&v_lds[0][0]));
    }
    t_last = wall_clock64();
  }

  if (stats != nullptr && tid == 0) {
    shplb_wg_stats rec;
    rec.xcc_id = uint32_t(my_xcd());
    rec.cu_id = (__builtin_amdgcn_s_getreg((16 - 1) << 11 | 0 << 6 | 4) >> 8) & 0xff; // HW_ID[15:8]
    rec.n_items = my_items;
    rec.cost_blocks = my_cost;
    rec.t_first = t_first;
    rec.t_last = t_last;
    stats[blockIdx.x] = rec;
  }
}

template <int BQ>
void launch_one(const Geometry& g, const void* q, const void* k, const void* v, const int64_t* sel_ptr,
                const int32_t* sel_idx, void* out, float* lse, shplb_wg_stats* stats,
                WorkQueues wq, SplitBuffers sb, int32_t n_wg, hipStream_t stream) {
  const float scale_log2 = g.scale * 1.4426950408889634f;
  hipLaunchKernelGGL((attn_kernel<BQ>), dim3(n_wg), dim3(2 * BQ), 0, stream, g.meta, g.st,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                     static_cast<const uint16_t*>(v), sel_ptr, sel_idx, static_cast<uint16_t*>(out), lse,
                     stats, wq, sb, g.total_tokens, scale_log2);
}

}  // namespace

int32_t launch_attention(const Geometry& g, const void* q, const void* k, const void* v,
                         const int64_t* sel_ptr, const int32_t* sel_idx, void* out, float* lse,
                         shplb_wg_stats* stats, WorkQueues wq, SplitBuffers sb, int32_t n_wg, hipStream_t stream) {
  if (g.meta.block == 128)
    launch_attention_pipe128(g, q, k, v, sel_ptr, sel_idx, out, lse, stats, wq, sb, n_wg, stream);
  else
    launch_one<64>(g, q, k, v, sel_ptr, sel_idx, out, lse, stats, wq, sb, n_wg, stream);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
