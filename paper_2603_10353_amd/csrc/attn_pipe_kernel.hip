// Software-pipelined block-sparse causal attention over per-row selected key blocks (gfx950).
//
// Work item = one (sequence, head, query block) row of the selection, or a piece of one.
// Persistent workgroups draw items from cost-descending queues through atomic tickets.
//
// Tiling (wave64, v_mfma_f32_32x32x16_bf16), for blocks of BQ = 128 or 64 tokens:
//   * a wave owns 32 query rows and keeps Q as MFMA B-operands in registers; a query block is
//     BQ/32 waves.  Block 128: 4 waves, two workgroups per compute unit; block 64: 2 waves, four
//     workgroups per compute unit.  Either way every SIMD holds two waves of different
//     workgroups, each with 256 registers, and one wave's softmax VALU work overlaps the other's
//     MFMAs;
//   * keys are streamed in tiles of KT = BQ/2 keys, two tiles per key block.  K and V rows go
//     from global memory straight into a double-buffered LDS stage (global_load_lds_dwordx4, no
//     staging registers, no LDS store instructions).  Rows are 256 bytes, unpadded; the 16-byte
//     chunk c of row r sits at chunk slot c ^ swz(r), which keeps both the K operand reads and
//     the V transpose reads free of bank conflicts;
//   * the first contraction is S^T = K Q^T (A = K from LDS by 16-byte reads), so a lane holds one
//     query column: the softmax max/sum are in-lane plus one exchange with lane^32, and the
//     probabilities feed the second contraction O^T += V^T P^T straight from registers (the key
//     order inside a 16-key MFMA step is permuted identically on both operands, which a sum over
//     keys does not see); V^T operands come from the LDS transpose read (ds_read_b64_tr_b16);
//   * the order of work inside a wave.  A step handles tile t's softmax and second contraction
//     and tile t+1's first contraction:
//
//       step t:  barrier                      K(t+1), V(t) resident; stages of K(t), V(t-1) free
//                copies K(t+2), V(t+1) start
//                the MFMAs of S(t+1), back to back; mask S(t+1) if it is the diagonal block
//                exp / bf16 pack / row sum of the probabilities of tile t (one run of VALU work);
//                if a row sum shows that the reference maximum was too low (rare): true
//                maximum of the tile, rescale O and l, probabilities again
//                the MFMAs of O += V(t)^T P(t)^T, back to back
//
//     so a wave alternates between blocks of MFMAs and a block of VALU work that depends
//     on none of the MFMAs in flight, and the two waves of a SIMD (of different workgroups,
//     unsynchronised) mostly find the other unit free.
//
// The two score buffers swap roles from step to step (the tile count is even, steps are
// issued in pairs).  LDS operands are fetched kLook groups ahead of their use.  Fully
// masked sub-tiles are computed like any other (their probabilities are exact zeros).
// With 64-token blocks a tile feeds half as many MFMAs per copy, barrier and item as with 128.
#include <type_traits>

#include "attn_common.h"

namespace shplb {
namespace {

template <int BQ>
__global__ __launch_bounds__(2 * BQ) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_pipe_kernel(SeqMeta meta, Strides st, const uint16_t* __restrict__ q,
                      const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                      const int64_t* __restrict__ sel_ptr, const int32_t* __restrict__ sel_idx,
                      uint16_t* __restrict__ out, float* __restrict__ lse,
                      shplb_wg_stats* __restrict__ stats, WorkQueues wq, SplitBuffers sb, int64_t total_tokens,
                      float scale_log2) {
  constexpr int NT = 1;                              // 32-query tiles per wave
  constexpr int kWaves = BQ / 32;
  constexpr int QW = 32;                             // query rows per wave
  constexpr int KT = BQ / 2;                         // keys per tile: two tiles per key block
  constexpr int MT = KT / 32;                        // 32-key MFMA tiles of a tile's scores
  constexpr int kTileBytes = KT * kRowBytes;
  constexpr int kRoundRows = 4 * kWaves;             // rows one round of copies moves (4 per wave)
  constexpr int kRounds = KT / kRoundRows;
  constexpr int kQK = 8 * MT;                        // MFMAs of a tile's first contraction, index 2*ks + mt (MT = 2) or ks
  constexpr int kPV = 4 * (KT / 16);                 // ... of its second, index 4*gq + dt
  constexpr int kLook = 8;             // LDS operand fetches run this many groups ahead
  constexpr float kSumLimit = 16.0f * MT * 256.0f;   // a lane's 16 MT probabilities of a tile can only sum to
                                                     // more if one of them exceeds 2^8

  __shared__ __attribute__((aligned(1024))) char k_lds[2][kTileBytes];
  __shared__ __attribute__((aligned(1024))) char v_lds[2][kTileBytes];
  __shared__ int32_t s_item;
  __shared__ int32_t s_flag;
  __shared__ int32_t s_merge[kDeferredMerges];   // items whose row this workgroup still has to combine

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hi = lane >> 5;
  const int64_t row_bytes = st.kv_t * 2;

  // ---- per-lane constants
  // copies: lane (r4 = lane>>4, slot = lane&15) of a wave fills, in round rd, LDS row
  // rd*kRoundRows + cp_row, slot `slot`, with the source chunk slot ^ swz(row).  Rounds of 8
  // rows alternate bit 3 of the row, which flips the low bit of the swizzle: two per-lane
  // source offsets cover all rounds.
  // K operand reads: lane (n, hi) reads row 32mt + n, chunk 2ks + hi.
  // V transpose reads: lane = 16*grp + 4e + a supplies the piece (key 16gq + 8half + 4hi + e,
  // dims 32dt + 16(grp&1) + 4a ..) and receives keys 4hi+0..3 (+8half, +16gq) of dim 32dt + n.
  const int cp_row = 4 * wave + (lane >> 4);
  const uint32_t cp_off0 = uint32_t(cp_row) * uint32_t(row_bytes) + (((lane & 15) ^ swz(cp_row)) << 4);
  const uint32_t cp_off1 = uint32_t(cp_row) * uint32_t(row_bytes) + (((lane & 15) ^ swz(cp_row) ^ 1) << 4);
  const int k_rd0 = n * kRowBytes + ((hi ^ swz(n)) << 4);
  const int tr_e = (lane >> 2) & 3, tr_a = lane & 3, tr_mh = (lane >> 4) & 1;
  int v_rd0[2];
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int r = 8 * half + 4 * hi + tr_e;
    v_rd0[half] = r * kRowBytes + (((2 * tr_mh + (tr_a >> 1)) ^ swz(r)) << 4) + 8 * (tr_a & 1);
  }
  const uint32_t k_stage0 = __builtin_amdgcn_readfirstlane(lds_offset_of(&k_lds[0][0]) + 4 * wave * kRowBytes);
  const uint32_t v_stage0 = __builtin_amdgcn_readfirstlane(lds_offset_of(&v_lds[0][0]) + 4 * wave * kRowBytes);

  // The two workgroups of a compute unit compete for every SIMD's issue slots, and left alone
  // one of them wins most of the time: workgroups were measured to get through 30-40% more or
  // fewer key blocks than the average in the same time.  The sum is what counts in the middle
  // of a launch, but near its end the slow workgroup of a pair holds its last item far longer
  // than planned and the launch waits for it.  So the pair takes turns: wave priority 1 for
  // one and 0 for the other, swapped every 2^kTurnShift ticks of the constant 100 MHz clock
  // (41 us), the first half of the grid against the second half (the dispatcher fills every
  // compute unit once before it places second workgroups; if it ever does not, two workgroups
  // merely swap in step and nothing is lost).  Progress per workgroup then stays within 6-7%
  // of the average and the idle tail of short launches shrinks (64K share of 8 heads: 6% of
  // the launch to 2-3%).
  constexpr int kTurnShift = 12;
  const uint32_t second_wg = blockIdx.x >= gridDim.x / 2;

  uint32_t my_items = 0, my_cost = 0;
  uint64_t t_first = 0, t_last = 0;
  const int home = my_xcd();
  int empty_mask = 0;                    // queues this workgroup has found empty (thread 0 only)
  int n_merge = 0;                       // rows whose last piece finished here; combined after the loop

  for (;;) {
    // A workgroup that owes as many merges as it can note stops taking items; the others carry on
    // (there are far fewer split rows in a launch than the workgroups together can note).
    if (n_merge == kDeferredMerges) break;
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
    const int n_tiles = n_sel * 2;                     // two 64-key tiles per 128-token block: always even
    if (n_sel <= 0) continue;
    if (my_items == 0) t_first = wall_clock64();
    my_items += 1;
    my_cost += uint32_t(n_sel);

    const char* k_head = reinterpret_cast<const char*>(k + int64_t(g) * st.kv_h);
    const char* v_head = reinterpret_cast<const char*>(v + int64_t(g) * st.kv_h);

    // Copy the K or V rows of tile t into LDS stage `stage`.
    auto issue = [&](const char* head, uint32_t stage0, int t, int stage, int j_raw) {
      const int j = min(max(j_raw, 0), nb - 1);
      // a sub-tile that starts past the end of a ragged last block is moved back onto the
      // last token: row offsets must stay non-negative (they are added unsigned)
      const int key_base = min(seq_begin + j * BQ + KT * (t & 1), seq_end - 1);
      const int last = seq_end - 1 - key_base;
      const char* tile = head + int64_t(key_base) * row_bytes;
      const uint32_t dst = stage0 + stage * kTileBytes;
      if (last >= KT - 1) {
#pragma unroll
        for (int rd = 0; rd < kRounds; ++rd) {
          const bool odd8 = ((rd * kRoundRows) >> 3) & 1;       // round starts at an odd multiple of 8 rows
          copy_g2l_16(tile + int64_t(rd * kRoundRows) * row_bytes, odd8 ? cp_off1 : cp_off0,
                      dst + rd * kRoundRows * kRowBytes);
        }
      } else {                                     // ragged: rows past the end re-read the last valid key (masked)
#pragma unroll
        for (int rd = 0; rd < kRounds; ++rd) {
          const int r = rd * kRoundRows + cp_row;
          const uint32_t off = uint32_t(min(r, last)) * uint32_t(row_bytes) + (((lane & 15) ^ swz(r)) << 4);
          copy_g2l_16(tile, off, dst + rd * kRoundRows * kRowBytes);
        }
      }
    };
    // selected block of tile pair b (tiles 2b, 2b+1); read one pair ahead of its first use so
    // that the scalar-memory latency never sits in front of a copy
    auto block_of = [&](int b) { return sel_idx[sel_begin + min(b, n_sel - 1)]; };
    int j0 = block_of(0), j1 = block_of(1);

    issue(k_head, k_stage0, 0, 0, j0);
    issue(v_head, v_stage0, 0, 0, j0);
    issue(k_head, k_stage0, 1, 1, j0);

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

    auto mask_scores = [&](f32x16 (&sc)[MT][NT], int t) {          // diagonal block: keys above the query
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        // key position minus query position, up to the part that depends on the register: taken
        // through an opaque move so that the 32 comparisons are made here, on the rare diagonal
        // tile, instead of being hoisted out of the item loop into 64 scalar registers of masks
        int d = KT * (t & 1) + 4 * hi - (wave * QW + 32 * nt + n);
        asm volatile("" : "+v"(d));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (d + (32 * mt + 8 * (r >> 2) + (r & 3)) > 0) sc[mt][nt][r] = -INFINITY;
      }
    };
    // mx[nt] = in-lane maximum of a tile's scores: raise the reference to it where it is higher
    auto settle_max = [&](float (&mx)[NT]) {
      {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const float m_new = fmaxf(m_ref[nt], pair_max(mx[nt]) * scale_log2);
          const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref[nt] - m_new);
          m_ref[nt] = m_new;
          l_run[nt] *= alpha;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[dt][nt][r] *= alpha;
        }
      }
    };

    auto read_k = [&](const char* kt, int gi) {       // operand of QK group gi = MT*ks + mt
      const int ks = gi / MT, mt = gi % MT;
      return *reinterpret_cast<const bf16x8*>(kt + (k_rd0 ^ (ks << 5)) + mt * 32 * kRowBytes);
    };
    // in-lane maximum of a tile's scores
    auto tile_max = [&](f32x16 (&sc)[MT][NT], float (&mx)[NT]) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if constexpr (MT == 2) {
          mx[nt] = fmaxf(sc[0][nt][0], sc[1][nt][0]);
#pragma unroll
          for (int r = 1; r < 16; ++r) mx[nt] = fmaxf(mx[nt], fmaxf(sc[0][nt][r], sc[1][nt][r]));
        } else {
          mx[nt] = sc[0][nt][0];
#pragma unroll
          for (int r = 1; r < 16; ++r) mx[nt] = fmaxf(mx[nt], sc[0][nt][r]);
        }
      }
    };
    auto read_v = [&](const char* vt, int gi) {       // operand of PV group gi = 4*gq + dt
      const int gq = gi >> 2, dt = gi & 3;
      const s16x4 lo = lds_read_tr16(vt + (v_rd0[0] ^ (dt << 6)) + gq * 16 * kRowBytes);
      const s16x4 up = lds_read_tr16(vt + (v_rd0[1] ^ (dt << 6)) + gq * 16 * kRowBytes);
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    // ---- prologue: S(0)
    f32x16 sc_a[MT][NT], sc_b[MT][NT];
    wait_vmem_all();
    __syncthreads();
    {
      const char* kt = k_lds[0];
      bf16x8 kf[kQK];
#pragma unroll
      for (int gi = 0; gi < kQK; ++gi) kf[gi] = read_k(kt, gi);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int r = 0; r < 16; ++r) sc_a[mt][nt][r] = 0.0f;
#pragma unroll
      for (int gi = 0; gi < kQK; ++gi)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          sc_a[gi % MT][nt] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[gi], qf[nt][gi / MT], sc_a[gi % MT][nt], 0, 0, 0);
      if (j0 == i) mask_scores(sc_a, 0);
      float mx[NT];
      tile_max(sc_a, mx);
      settle_max(mx);
    }

    // One step: tile t's softmax and PV from sc_cur, tile t+1's scores into sc_nxt.
    // jv / jk: selected blocks of tiles t+1 and t+2.
    auto step = [&](auto has_next_c, f32x16 (&sc_cur)[MT][NT], f32x16 (&sc_nxt)[MT][NT], int t, int jv, int jk) {
      constexpr bool kHasNext = decltype(has_next_c)::value;
      // Take turns with the other workgroup of this compute unit (see kTurnShift).
      if (((uint32_t(wall_clock64()) >> kTurnShift) & 1) ^ second_wg) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
      wait_vmem_all();                  // own copies of K(t+1), V(t) have landed
      __syncthreads();                  // everyone's have; stages of K(t) and V(t-1) are free
      if (t + 2 < n_tiles) issue(k_head, k_stage0, t + 2, t & 1, jk);
      if (kHasNext) issue(v_head, v_stage0, t + 1, (t + 1) & 1, jv);

      const char* kn = k_lds[(t + 1) & 1];
      const char* vc = v_lds[t & 1];
      float m_use[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) m_use[nt] = m_ref[nt] == -INFINITY ? 0.0f : m_ref[nt];

      bf16x8 kf[kQK], vf[kPV];
      uint32_t pk[NT][MT][8];
      float rs0[NT], rs1[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) rs0[nt] = rs1[nt] = 0.0f;
      if (kHasNext) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc_nxt[mt][nt][r] = 0.0f;
      }

      // ---- S(t+1): its MFMAs back to back (the operands of the second contraction are
      // fetched behind the last K operands)
      static_assert(kLook <= kQK && kLook <= kPV, "operand lookahead longer than a contraction");
      if (kHasNext) {
#pragma unroll
        for (int gi = 0; gi < kLook; ++gi) kf[gi] = read_k(kn, gi);
      } else {
#pragma unroll
        for (int gi = 0; gi < kLook; ++gi) vf[gi] = read_v(vc, gi);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (kHasNext) {
#pragma unroll
        for (int gi = 0; gi < kQK; ++gi) {
          if (gi + kLook < kQK) kf[gi + kLook] = read_k(kn, gi + kLook);
          else vf[gi + kLook - kQK] = read_v(vc, gi + kLook - kQK);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            sc_nxt[gi % MT][nt] =
                __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[gi], qf[nt][gi / MT], sc_nxt[gi % MT][nt], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (jv == i) mask_scores(sc_nxt, t + 1);
      }

      // ---- probabilities of tile t, in one run of VALU work: the S(t+1) MFMAs of this wave
      // are still in flight and the other wave of the SIMD is usually inside an MFMA block.
      // (Spread between the MFMAs above, the same instructions make the kernel 2-4% slower.)
      auto probabilities = [&]() {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          m_use[nt] = m_ref[nt] == -INFINITY ? 0.0f : m_ref[nt];
          rs0[nt] = rs1[nt] = 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8 * MT; ++u) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const int mt = u >> 3, r = 2 * (u & 7);
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc_cur[mt][nt][r], scale_log2, -m_use[nt]));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc_cur[mt][nt][r + 1], scale_log2, -m_use[nt]));
            pk[nt][mt][u & 7] = pack_bf16(p0, p1);
            // row sum of the rounded probabilities (what the second contraction multiplies with)
            if (u & 1) rs1[nt] = dot2_ones(pk[nt][mt][u & 7], rs1[nt]);
            else rs0[nt] = dot2_ones(pk[nt][mt][u & 7], rs0[nt]);
          }
        }
      };
      probabilities();
      // The reference m_ref was fixed by earlier tiles.  It is too low for this tile exactly
      // when a probability came out large, and then the tile's row sum is large: no maximum
      // over the scores is needed to notice.  In that (rare) case take the tile's true
      // maximum, raise the reference, rescale O and l, and redo the tile's probabilities.
      {
        bool big = false;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) big = big || !(rs0[nt] + rs1[nt] <= kSumLimit);
        if (__any(big)) {
          float mx[NT];
          tile_max(sc_cur, mx);
          settle_max(mx);
          probabilities();
        }
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) l_run[nt] += rs0[nt] + rs1[nt];
      __builtin_amdgcn_sched_barrier(0);

      // ---- O^T += V(t)^T P(t)^T: its MFMAs back to back
#pragma unroll
      for (int gi = 0; gi < kPV; ++gi) {
        if (gi + kLook < kPV) vf[gi + kLook] = read_v(vc, gi + kLook);
        const int gq = gi >> 2, dt = gi & 3;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const u32x4 w = {pk[nt][gq >> 1][4 * (gq & 1)], pk[nt][gq >> 1][4 * (gq & 1) + 1],
                           pk[nt][gq >> 1][4 * (gq & 1) + 2], pk[nt][gq >> 1][4 * (gq & 1) + 3]};
          acc_o[dt][nt] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[gi], __builtin_bit_cast(bf16x8, w), acc_o[dt][nt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };

    for (int b = 0; b + 1 < n_sel; ++b) {
      const int j2 = block_of(b + 2);
      step(std::true_type{}, sc_a, sc_b, 2 * b, j0, j1);
      step(std::true_type{}, sc_b, sc_a, 2 * b + 1, j1, j1);
      j0 = j1;
      j1 = j2;
    }
    step(std::true_type{}, sc_a, sc_b, n_tiles - 2, j0, j0);
    step(std::false_type{}, sc_b, sc_a, n_tiles - 1, j0, j0);

    // ---- normalise and store: lane holds, for its query, dims 32dt + 8(r/4) + 4hi + (r%4)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const float l_tot = pair_sum(l_run[nt]);
      if (slot >= 0) {
        // a piece of a split row: O and l as they stand (relative to 2^m_ref), for merge_row()
        const int q_in = wave * QW + 32 * nt + n;
        float* part = sb.part_o + int64_t(slot) * kSlotFloatsO;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            float* dst = part + slot_chunk(wave * NT + nt, dt, rq, lane);
            slot_store(dst, acc_o[dt][nt][4 * rq], acc_o[dt][nt][4 * rq + 1]);
            slot_store(dst + 2, acc_o[dt][nt][4 * rq + 2], acc_o[dt][nt][4 * rq + 3]);
          }
        if (hi == 0) {
          float* ml = sb.part_ml + int64_t(slot) * kSlotFloatsML;
          slot_store1(ml + q_in, m_ref[nt]);
          slot_store1(ml + 128 + q_in, l_tot);
        }
      } else {
        // The two lanes of a query hold alternating runs of four dims (8 bytes as bf16).  They trade
        // runs so that each ends up with eight consecutive dims: the lower lane takes both halves of
        // the even runs, the upper lane of the odd ones, and a row goes out in 16-byte stores, two
        // lanes per 32 bytes, instead of 8-byte stores scattered over 64 rows.
        const float inv = 1.0f / l_tot;
        const bool valid = q_tok[nt] < seq_end;
        uint16_t* dst = out + int64_t(valid ? q_tok[nt] : seq_end - 1) * st.q_t + int64_t(h) * st.q_h + 8 * hi;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int rp = 0; rp < 2; ++rp) {
            const int ra = 8 * rp, rb = 8 * rp + 4;      // first accumulator of the even and of the odd run
            uint32_t e0 = pack_bf16(acc_o[dt][nt][ra] * inv, acc_o[dt][nt][ra + 1] * inv);
            uint32_t e1 = pack_bf16(acc_o[dt][nt][ra + 2] * inv, acc_o[dt][nt][ra + 3] * inv);
            uint32_t o0 = pack_bf16(acc_o[dt][nt][rb] * inv, acc_o[dt][nt][rb + 1] * inv);
            uint32_t o1 = pack_bf16(acc_o[dt][nt][rb + 2] * inv, acc_o[dt][nt][rb + 3] * inv);
            swap_halves(e0, o0);                         // lower lane: even run of both; upper lane: odd run of both
            swap_halves(e1, o1);
            if (valid) *reinterpret_cast<u32x4*>(dst + 32 * dt + 16 * rp) = u32x4{e0, e1, o0, o1};
          }
        if (valid && lse != nullptr && hi == 0)
          lse[int64_t(h) * total_tokens + q_tok[nt]] =
              (m_ref[nt] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
      }
    }
    if (slot >= 0) {
      // a piece: count it; if it completes its row, note the row for the merge after the loop
      if (count_piece(sb, item->pieces, item->split_index, &s_flag)) {
        if (tid == 0) s_merge[n_merge] = pos;
        n_merge += 1;
      }
    }
    t_last = wall_clock64();
  }

  // ---- rows whose pieces are all done and whose last piece this workgroup computed
  for (int x = 0; x < n_merge; ++x) {
    __syncthreads();                                   // s_merge as thread 0 left it
    const ItemRec* item = wq.items + s_merge[x];
    int s, h, i, nb;
    decode_row(meta, item->row, s, h, i, nb);
    const int q0 = meta.tok_begin[s] + i * BQ;
    merge_row<BQ, 2 * BQ>(sb, item->pieces, item->first_slot, out + int64_t(q0) * st.q_t + int64_t(h) * st.q_h,
                          st.q_t, lse != nullptr ? lse + int64_t(h) * total_tokens + q0 : nullptr,
                          min(BQ, meta.tok_begin[s + 1] - q0), reinterpret_cast<float*>(&k_lds[0][0]),
                          reinterpret_cast<float*>(&v_lds[0][0]));
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
                const int32_t* sel_idx, void* out, float* lse, shplb_wg_stats* stats, WorkQueues wq,
                SplitBuffers sb, int32_t n_wg, hipStream_t stream) {
  const float scale_log2 = g.scale * 1.4426950408889634f;
  hipLaunchKernelGGL((attn_pipe_kernel<BQ>), dim3(n_wg), dim3(2 * BQ), 0, stream, g.meta, g.st,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                     static_cast<const uint16_t*>(v), sel_ptr, sel_idx, static_cast<uint16_t*>(out), lse,
                     stats, wq, sb, g.total_tokens, scale_log2);
}

}  // namespace

int32_t launch_attention(const Geometry& g, const void* q, const void* k, const void* v,
                         const int64_t* sel_ptr, const int32_t* sel_idx, void* out, float* lse,
                         shplb_wg_stats* stats, WorkQueues wq, SplitBuffers sb, int32_t n_wg, hipStream_t stream) {
  if (g.meta.block == 128) launch_one<128>(g, q, k, v, sel_ptr, sel_idx, out, lse, stats, wq, sb, n_wg, stream);
  else launch_one<64>(g, q, k, v, sel_ptr, sel_idx, out, lse, stats, wq, sb, n_wg, stream);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
