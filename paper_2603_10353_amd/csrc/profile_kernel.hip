// Recovery profiles (paper Section 2.4), two dense causal passes that are not on the hot path:
//
//  * mass_kernel: at block granularity, the attention weight every query block puts on every key
//    block of the causal triangle, under full attention,
//      mass[s][h][i][j] = 1/n_i * sum over the valid queries t of block i, keys u of block j, u <= t,
//                         of softmax_t(q_t . k_u * scale)                    (j <= i; rows sum to 1)
//    Sorted per row and accumulated it gives the recovery curves that budget shifting consumes,
//    and summed over a selection it says how much of the attention that selection keeps.
//  * token_recovery_kernel: at the paper's own granularity, for every query token the sum of its
//    k largest attention weights, for up to eight budgets k at once.
//
// Both share the first contraction of the attention kernels (64-key K tiles copied global->LDS
// into swizzled 256-byte rows, S^T = K Q^T with Q in registers, a lane owns one query column) and
// have no second one.  One workgroup = one (sequence, head, query block) row, all key blocks
// 0 .. i, in several sweeps over the row's keys; the scores are recomputed in every sweep (the
// triangle of probabilities does not fit anywhere).  Rows are launched heaviest first (largest i
// first), so the tail of the launch is short rows.
#include "attn_common.h"

namespace shplb {
namespace {

// One (sequence, head, query block) row swept over its keys: tile copies, Q fragments, raw scores.
template <int BQ>
struct DenseRow {
  static constexpr int kWaves = BQ / 32;
  static constexpr int SUB = BQ / kKeysPerTile;            // 64-key tiles per key block
  static constexpr int kRoundRows = 4 * kWaves;
  static constexpr int kRounds = kKeysPerTile / kRoundRows;

  int s, h, i, nb, tid, lane, wave, n, hi;
  int seq_begin, seq_end, n_tiles, q_tok, n_valid;
  int cp_row, k_rd0;
  int step;                                         // tiles handled so far over all sweeps: stage = step & 1
  uint32_t k_stage0;
  int64_t row_bytes;
  const char* k_head;
  const char* k_lds;                                // two stages of kTileBytes
  bf16x8 qf[8];                                     // B operand of S^T = K Q^T: dims 16ks + 8hi.. of the lane's query

  // blockIdx.x = level * (sequences * heads) + (s * heads + h); level 0 is the last query block.
  // False: this sequence of a varlen batch has no such block.
  __device__ __forceinline__ bool init(const SeqMeta& meta, const Strides& st, const uint16_t* __restrict__ q,
                                       const uint16_t* __restrict__ k, int max_nb, const char* lds) {
    const int per_level = meta.n_seq * meta.n_q_heads;
    const int level = blockIdx.x / per_level, sh = blockIdx.x - level * per_level;
    s = sh / meta.n_q_heads;
    h = sh - s * meta.n_q_heads;
    nb = meta.blk_begin[s + 1] - meta.blk_begin[s];
    i = max_nb - 1 - level;
    if (i >= nb) return false;
    tid = threadIdx.x;
    lane = tid & 63;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    n = lane & 31;
    hi = lane >> 5;
    seq_begin = meta.tok_begin[s];
    seq_end = meta.tok_begin[s + 1];
    n_tiles = (i + 1) * SUB;
    row_bytes = st.kv_t * 2;
    k_head = reinterpret_cast<const char*>(k + int64_t(kv_head_of(meta, h)) * st.kv_h);
    k_lds = lds;
    cp_row = 4 * wave + (lane >> 4);
    k_rd0 = n * kRowBytes + ((hi ^ swz(n)) << 4);
    k_stage0 = __builtin_amdgcn_readfirstlane(lds_offset_of(lds) + 4 * wave * kRowBytes);
    step = 0;
    q_tok = seq_begin + i * BQ + wave * 32 + n;
    n_valid = min(BQ, seq_end - seq_begin - i * BQ);
    const uint16_t* src = q + int64_t(min(q_tok, seq_end - 1)) * st.q_t + int64_t(h) * st.q_h + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
    return true;
  }
  __device__ __forceinline__ bool live() const { return q_tok < seq_end; }   // not a padding query of a ragged last block

  // Copy the 64 keys of tile `it` (block it / SUB) into LDS stage `buf`.
  __device__ __forceinline__ void issue_tile(int it, int buf) const {
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
      // (the LDS base goes into M0: a scalar, said explicitly because it is derived from struct members)
      copy_g2l_16(k_tile, off, __builtin_amdgcn_readfirstlane(k_stage0 + buf * kTileBytes + rd * kRoundRows * kRowBytes));
    }
  }

  // raw scores (q . k, unscaled) of tile `it` from stage `buf`; on the diagonal block the keys above the
  // query are set to -inf (only there: the test is uniform, so other tiles pay nothing for it)
  __device__ __forceinline__ void scores_of(int it, int buf, f32x16 (&sc)[2]) const {
    const char* kt = k_lds + buf * kTileBytes;
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
  }

  // One sweep over the row's tiles: per_tile(it, sc) sees the raw scores of tile `it`.  The first tile
  // must be on its way into stage step & 1; with `another` the last iteration starts the first tile
  // of the next sweep.  (A sweep that is the kernel's last must not: a copy that lands after the
  // workgroup has ended writes into LDS that is no longer its own.)
  template <class F>
  __device__ __forceinline__ void sweep(bool another, F&& per_tile) {
    for (int it = 0; it < n_tiles; ++it, ++step) {
      wait_vmem_all();
      __syncthreads();
      if (it + 1 < n_tiles) issue_tile(it + 1, (step + 1) & 1);
      else if (another) issue_tile(0, (step + 1) & 1);
      f32x16 sc[2];
      scores_of(it, step & 1, sc);
      per_tile(it, sc);
    }
  }

  // First sweep: log2 of the softmax denominator of the lane's query, exact fp32 statistics (nothing
  // rounded to bf16).  The sum runs against a reference exponent that is only raised when a tile's
  // maximum exceeds it by more than 2^8 (then the sum so far is rescaled): exact in real arithmetic,
  // and most tiles cost one fused multiply-add, one exponential and one addition per score, plus the
  // maximum.  The two lanes of a query hold disjoint halves of its keys and are merged at the end.
  __device__ __forceinline__ float log2_denominator(float scale_log2) {
    float m_run = -INFINITY, l_run = 0.0f;
    sweep(true, [&](int, f32x16 (&sc)[2]) {
      float mx = fmaxf(sc[0][0], sc[1][0]);
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(sc[0][r], sc[1][r]));
      mx *= scale_log2;
      if (mx > m_run + kRescaleSlack) {             // per lane: a lane's reference follows its own keys
        l_run *= m_run == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(m_run - mx);
        m_run = mx;
      }
      if (m_run != -INFINITY) {                     // all keys of the lane masked so far: nothing to add
        float sum0 = 0.0f, sum1 = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          sum0 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0][r], scale_log2, -m_run));
          sum1 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[1][r], scale_log2, -m_run));
        }
        l_run += sum0 + sum1;
      }
    });
    float m_lo, m_hi, l_lo, l_hi;
    pair_values(m_run, m_lo, m_hi);
    pair_values(l_run, l_lo, l_hi);
    const float m_all = fmaxf(m_lo, m_hi);
    const float l_all = (m_lo == -INFINITY ? 0.0f : l_lo * __builtin_amdgcn_exp2f(m_lo - m_all)) +
                        (m_hi == -INFINITY ? 0.0f : l_hi * __builtin_amdgcn_exp2f(m_hi - m_all));
    return m_all + __builtin_amdgcn_logf(l_all);    // v_log_f32 is a base-2 logarithm
  }
};

// Two sweeps: the softmax denominators, then the probabilities exp2(s - lse) summed over the lane's
// keys, the tiles of a key block, the wave (shuffles) and the waves (LDS, fixed order): one number
// per key block, bit-identical from run to run.
template <int BQ>
__global__ __launch_bounds__(2 * BQ) void mass_kernel(SeqMeta meta, Strides st, const uint16_t* __restrict__ q,
                                                      const uint16_t* __restrict__ k, float* __restrict__ mass,
                                                      int max_nb, float scale_log2) {
  using Row = DenseRow<BQ>;
  __shared__ __attribute__((aligned(1024))) char k_lds[2][kTileBytes];
  __shared__ float s_part[2][Row::kWaves];

  Row row;
  if (!row.init(meta, st, q, k, max_nb, &k_lds[0][0])) return;
  row.issue_tile(0, 0);
  float* out_row = mass + meta.score_off[row.s] + (int64_t(row.h) * row.nb + row.i) * row.nb;
  const float lse2 = row.log2_denominator(scale_log2);
  const bool live = row.live();
  const float per_query = 1.0f / float(row.n_valid);

  float acc = 0.0f;
  row.sweep(false, [&](int it, f32x16 (&sc)[2]) {
    const int j = it / Row::SUB, sub = it - j * Row::SUB;
    if (sub == 0 && j > 0 && row.tid == 0) {        // block j-1 is complete and visible: fixed-order sum
      float tot = 0.0f;
#pragma unroll
      for (int w = 0; w < Row::kWaves; ++w) tot += s_part[(j - 1) & 1][w];
      out_row[j - 1] = tot * per_query;
    }
    float sum0 = 0.0f, sum1 = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sum0 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0][r], scale_log2, -lse2));
      sum1 += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[1][r], scale_log2, -lse2));
    }
    acc += live ? sum0 + sum1 : 0.0f;
    if (sub == Row::SUB - 1) {
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d);
      if (row.lane == 0) s_part[j & 1][row.wave] = acc;
      acc = 0.0f;
    }
  });
  __syncthreads();
  if (row.tid == 0) {
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < Row::kWaves; ++w) tot += s_part[row.i & 1][w];
    out_row[row.i] = tot * per_query;
  }
}

struct TokenBudgets {
  int32_t k[SHPLB_MAX_TOKEN_BUDGETS];
};

// Sum of the k largest attention weights of every query, for M budgets k at once.
//
// A weight is p = 2^-y with y = log2(denominator) - score * scale * log2(e) >= 0, so the k largest
// weights are the k smallest y, and the bit pattern of a non-negative float orders like the float.
// After the denominators (first sweep) the k-th smallest y of every query is found bit by bit, one
// sweep per bit: v grows from 0; with probe = v | bit, the number of the query's keys with y < probe
// is counted (a compare and an add-with-carry per score and budget; the two lanes that share a query
// add their counts); fewer than k means the k-th smallest is at least probe.  A count of exactly k
// settles the query early (its k best are the keys below probe), and the search ends when every query
// of the workgroup is settled; with distinct weights that happens once the probes separate the k-th
// from the (k+1)-th, in 20 to 25 sweeps instead of 31.  A last sweep sums the weights below v and
// adds the remainder of the budget at the weight of v itself (ties at the k-th place).  A y that
// rounding made slightly negative (one dominant key, p = 1 + a few ulp) is negative as an integer
// too and counts as smallest, which it is.  Queries that see at most k keys recover exactly 1.
template <int BQ, int M>
__global__ __launch_bounds__(2 * BQ) void token_recovery_kernel(SeqMeta meta, Strides st,
                                                                const uint16_t* __restrict__ q,
                                                                const uint16_t* __restrict__ k,
                                                                float* __restrict__ recovery, TokenBudgets budgets,
                                                                int n_out, int max_nb, float scale_log2,
                                                                int total_tokens) {
  using Row = DenseRow<BQ>;
  __shared__ __attribute__((aligned(1024))) char k_lds[2][kTileBytes];
  __shared__ int s_open[2][Row::kWaves];

  Row row;
  if (!row.init(meta, st, q, k, max_nb, &k_lds[0][0])) return;
  row.issue_tile(0, 0);
  const float lse2 = row.log2_denominator(scale_log2);
  const float neg_scale = -scale_log2;
  const int visible = row.q_tok - row.seq_begin + 1;          // keys the lane's query sees

  int v[M], want[M];
  bool settled[M];
#pragma unroll
  for (int b = 0; b < M; ++b) {
    want[b] = budgets.k[b];
    v[b] = 0;
    settled[b] = !row.live() || visible <= want[b];           // nothing to search
  }

  for (int bit = 30, round = 0;; --bit, ++round) {
    bool open = false;
#pragma unroll
    for (int b = 0; b < M; ++b) open |= !settled[b];
    // does any query of the workgroup still search?  (two flag sets: a wave may write the next
    // round's flag while another still reads this round's; a sweep's barriers separate the rounds)
    if (row.lane == 0) s_open[round & 1][row.wave] = 0;
    if (__any(open) && row.lane == 0) s_open[round & 1][row.wave] = 1;
    __syncthreads();
    int any_open = 0;
#pragma unroll
    for (int w = 0; w < Row::kWaves; ++w) any_open |= s_open[round & 1][w];
    if (!any_open || bit < 0) break;

    int probe[M], below[M];
#pragma unroll
    for (int b = 0; b < M; ++b) {
      probe[b] = v[b] | (1 << bit);
      below[b] = 0;
    }
    row.sweep(true, [&](int, f32x16 (&sc)[2]) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int y = __float_as_int(__builtin_fmaf(sc[mt][r], neg_scale, lse2));   // masked: +inf, above every probe
#pragma unroll
          for (int b = 0; b < M; ++b) below[b] += y < probe[b] ? 1 : 0;
        }
    });
#pragma unroll
    for (int b = 0; b < M; ++b) {
      float lo, up;
      pair_values(__int_as_float(below[b]), lo, up);
      const int cnt = __float_as_int(lo) + __float_as_int(up);
      if (!settled[b]) {
        if (cnt <= want[b]) v[b] = probe[b];
        if (cnt == want[b]) settled[b] = true;
      }
    }
  }

  float sum[M];
  int below[M];
#pragma unroll
  for (int b = 0; b < M; ++b) {
    sum[b] = 0.0f;
    below[b] = 0;
  }
  row.sweep(false, [&](int, f32x16 (&sc)[2]) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float yf = __builtin_fmaf(sc[mt][r], neg_scale, lse2);
        const float p = __builtin_amdgcn_exp2f(-yf);
        const int y = __float_as_int(yf);
#pragma unroll
        for (int b = 0; b < M; ++b) {
          sum[b] += y < v[b] ? p : 0.0f;
          below[b] += y < v[b] ? 1 : 0;
        }
      }
  });
  if (!row.live()) return;
#pragma unroll
  for (int b = 0; b < M; ++b) {
    float lo, up;
    pair_values(__int_as_float(below[b]), lo, up);
    const int rest = want[b] - (__float_as_int(lo) + __float_as_int(up));
    float r = pair_sum(sum[b]);
    if (rest > 0) r += float(rest) * __builtin_amdgcn_exp2f(-__int_as_float(v[b]));
    if (visible <= want[b]) r = 1.0f;
    if (b < n_out && row.hi == 0)
      recovery[(int64_t(b) * meta.n_q_heads + row.h) * total_tokens + row.q_tok] = r;
  }
}

template <int BQ, int M>
void launch_token_recovery_as(const Geometry& g, const uint16_t* q, const uint16_t* k, float* recovery,
                              const TokenBudgets& budgets, int n_out, uint32_t n_wg, hipStream_t stream) {
  hipLaunchKernelGGL((token_recovery_kernel<BQ, M>), dim3(n_wg), dim3(2 * BQ), 0, stream, g.meta, g.st, q, k,
                     recovery, budgets, n_out, g.max_nb, g.scale * 1.4426950408889634f, int(g.total_tokens));
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

int32_t launch_token_recovery(const Geometry& g, const void* q, const void* k, const int32_t* budgets,
                              int32_t n_budgets, float* recovery, hipStream_t stream) {
  const SeqMeta& m = g.meta;
  const int64_t n_wg = int64_t(g.max_nb) * m.n_seq * m.n_q_heads;
  if (n_wg > 0x7fffffff) return SHPLB_E_UNSUPPORTED;
  TokenBudgets kb;
  for (int b = 0; b < SHPLB_MAX_TOKEN_BUDGETS; ++b) kb.k[b] = budgets[std::min(b, n_budgets - 1)];
  const uint16_t* qp = static_cast<const uint16_t*>(q);
  const uint16_t* kp = static_cast<const uint16_t*>(k);
  const uint32_t wg = uint32_t(n_wg);
  const int width = n_budgets <= 1 ? 1 : n_budgets <= 2 ? 2 : n_budgets <= 4 ? 4 : 8;
  if (m.block == 128) {
    if (width == 1) launch_token_recovery_as<128, 1>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
    else if (width == 2) launch_token_recovery_as<128, 2>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
    else if (width == 4) launch_token_recovery_as<128, 4>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
    else launch_token_recovery_as<128, 8>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
  } else {
    if (width == 1) launch_token_recovery_as<64, 1>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
    else if (width == 2) launch_token_recovery_as<64, 2>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
    else if (width == 4) launch_token_recovery_as<64, 4>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
    else launch_token_recovery_as<64, 8>(g, qp, kp, recovery, kb, n_budgets, wg, stream);
  }
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
