// Per-head top-k key-block selection: one wavefront per (sequence, head, query block) row.
#include <type_traits>

#include "shplb_internal.h"

namespace shplb {
namespace {

// Monotone map float -> uint32 (larger float = larger key); +0 and -0 coincide.
__device__ __forceinline__ uint32_t order_key(float x) {
  x += 0.0f;                                   // -0 -> +0
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ int popc64(uint64_t m) { return __builtin_popcountll(m); }

// base + the number of set bits of m below this lane's own (v_mbcnt_lo, v_mbcnt_hi).
__device__ __forceinline__ int rank_in(uint64_t m, int base) {
  return int(__builtin_amdgcn_mbcnt_hi(uint32_t(m >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(m), uint32_t(base))));
}

// Maximum over the 64 lanes, as a scalar.  Four data-parallel-primitive steps make every lane of a
// row of 16 hold its row's maximum (exchange inside pairs, inside quads, mirror inside 8, mirror
// inside 16), then one lane per row is read: no LDS round trips, unlike six shuffle steps.
__device__ __forceinline__ uint32_t wave_max(uint32_t x) {
  auto dpp = [](uint32_t v, auto ctrl) {
    return uint32_t(__builtin_amdgcn_update_dpp(0, int(v), decltype(ctrl)::value, 0xf, 0xf, false));
  };
  x = max(x, dpp(x, std::integral_constant<int, 0xb1>{}));    // quad_perm [1,0,3,2]
  x = max(x, dpp(x, std::integral_constant<int, 0x4e>{}));    // quad_perm [2,3,0,1]
  x = max(x, dpp(x, std::integral_constant<int, 0x141>{}));   // row_half_mirror
  x = max(x, dpp(x, std::integral_constant<int, 0x140>{}));   // row_mirror
  const uint32_t a = __builtin_amdgcn_readlane(int(x), 0), b = __builtin_amdgcn_readlane(int(x), 16);
  const uint32_t c = __builtin_amdgcn_readlane(int(x), 32), d = __builtin_amdgcn_readlane(int(x), 48);
  return max(max(a, b), max(c, d));
}

// The row keeps block 0 and block i, then the `want` best of the candidates 1..i-1
// under the total order (score descending, index ascending).  The wave finds the
// want-th largest key t by a bitwise search (largest t with count(key >= t) >= want;
// at most 32 steps, usually about a dozen), takes every key > t, and fills the
// remainder with the lowest-index keys equal to t.  Output is written in ascending
// block order.
//
// SLOTS * 64 > i: lane l holds the candidates l, 64 + l, ... in SLOTS registers.  The body is
// instantiated for 2, 4, 8, ... slots and a row takes the smallest that holds it, so that
// every loop over the slots is unrolled without a test per slot and short rows (the early
// query blocks of every head) do not pay for long ones.
template <int SLOTS>
__device__ __forceinline__ void select_row(const float* __restrict__ srow, int32_t* __restrict__ out, int i,
                                           int want, int lane) {
  if (want >= i - 1) {                          // budget covers every candidate
#pragma unroll
    for (int c = 0; c < SLOTS; ++c) {
      const int j = c * 64 + lane;
      if (j >= 1 && j < i) out[j] = j;
    }
    return;
  }

  // All loads of the row are issued before the first is used (the index is clamped to the diagonal
  // entry, which exists, instead of branching around the load: a branch per slot makes every load
  // wait for the one before it, and a row of 1024 scores then costs sixteen memory round trips).
  float raw[SLOTS];
#pragma unroll
  for (int c = 0; c < SLOTS; ++c) raw[c] = srow[min(c * 64 + lane, i)];
  uint32_t key[SLOTS];
#pragma unroll
  for (int c = 0; c < SLOTS; ++c) {
    const int j = c * 64 + lane;
    key[c] = (j >= 1 && j < i) ? order_key(raw[c]) : 0u;   // 0 is below every real key (keys of finite floats are > 0)
  }

  // Scores of both signs are the rule, and the keys of the two signs lie far apart (the keys of small
  // magnitudes of either sign are the ones near the middle of the range), so a search over both would
  // spend its first steps on sign and exponent bits that split off nothing.  The want-th largest key is
  // non-negative if at least `want` keys are, else negative: one count decides, and the search is
  // confined to that sign.
  constexpr uint32_t kSign = 0x80000000u;
  int n_pos = 0;
#pragma unroll
  for (int c = 0; c < SLOTS; ++c) n_pos += popc64(__ballot(key[c] >= kSign));
  const bool among_pos = want <= n_pos;
  // All keys of that sign lie between its smallest and its largest, so t shares their common leading
  // bits (for scores of similar magnitude: most of the exponent); the search starts below them.  It
  // ends early when a probe splits off exactly `want` keys: those are the selection, whatever the
  // lower bits of t would be.
  uint32_t kmax = 0, kmin = 0xffffffffu;
#pragma unroll
  for (int c = 0; c < SLOTS; ++c) {
    const bool in = among_pos ? key[c] >= kSign : key[c] - 1u < kSign - 1u;   // (the 0 of an empty slot is in neither)
    if (in) {
      kmax = max(kmax, key[c]);
      kmin = min(kmin, key[c]);
    }
  }
  kmax = wave_max(kmax);
  kmin = ~wave_max(~kmin);
  uint32_t differ = kmax ^ kmin;
  uint32_t t = kmax;                            // all keys of the sign equal: ties only
  // Kept up to date during the search, so that no counting pass is needed after it:
  // at_least = count(key >= t) (>= want), above = count(key >= the lowest rejected probe) (< want);
  // after bit 0 the lowest rejected probe is t + 1, so above = count(key > t).  Keys of the other sign
  // are below every probe (negative ones) or above every probe (non-negative ones, counted from the start).
  int at_least = among_pos ? n_pos : i - 1, above = among_pos ? 0 : n_pos;
  bool exact = false;                           // a probe split off exactly `want` keys: no ties to ration
  if (n_pos == want) {                          // the non-negative keys are the selection
    t = kSign;
    exact = true;
    differ = 0;
  } else {
    // Keys are taken relative to the smallest of their sign (keys below it, and the 0 of empty slots,
    // become 0: a subtraction that saturates).  The order is the same, and the leading bits of the
    // largest key now count the exponents the keys really span instead of all the bits from the first
    // one in which two of them differ: about two steps fewer on pooled scores.
    const uint32_t shift = kmin - 1u;
#pragma unroll
    for (int c = 0; c < SLOTS; ++c) key[c] = __builtin_elementwise_sub_sat(key[c], shift);
    kmax -= shift;
    differ = kmax ^ 1u;                         // the smallest key is now 1
    t = kmax;
  }
  if (differ != 0) {
    const int top = 31 - __builtin_clz(differ);  // highest bit in which two candidates differ
    t = top == 31 ? 0u : kmax & ~((2u << top) - 1u);
    for (int bit = top; bit >= 0; --bit) {
      const uint32_t probe = t | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int c = 0; c < SLOTS; ++c) cnt += popc64(__ballot(key[c] >= probe));
      if (cnt == want) {
        t = probe;                              // the keys >= probe are exactly the selection
        exact = true;
        break;
      }
      if (cnt > want) {
        t = probe;
        at_least = cnt;
      } else {
        above = cnt;
      }
    }
  }

  int written = 0, ties_seen = 0;
  if (exact || at_least == want) {              // every key >= t is wanted (the usual case: no surplus ties)
#pragma unroll
    for (int c = 0; c < SLOTS; ++c) {
      const bool take = key[c] >= t;
      const uint64_t take_mask = __ballot(take);
      if (take) out[rank_in(take_mask, 1 + written)] = c * 64 + lane;
      written += popc64(take_mask);
    }
    return;
  }
  const int ties_wanted = want - above;         // >= 1 by construction of t
#pragma unroll
  for (int c = 0; c < SLOTS; ++c) {
    const bool is_tie = key[c] == t;
    const uint64_t tie_mask = __ballot(is_tie);
    const int tie_rank = rank_in(tie_mask, ties_seen);
    const bool take = key[c] > t || (is_tie && tie_rank < ties_wanted);
    const uint64_t take_mask = __ballot(take);
    if (take) out[rank_in(take_mask, 1 + written)] = c * 64 + lane;
    written += popc64(take_mask);
    ties_seen += popc64(tie_mask);
  }
}

// One wavefront per row; MAX_SLOTS * 64 >= number of blocks of the longest sequence.
template <int MAX_SLOTS>
__global__ __launch_bounds__(256) void select_kernel(
    SeqMeta meta, const float* __restrict__ scores, const int64_t* __restrict__ sel_ptr,
    int32_t* __restrict__ sel_idx, int32_t rows) {
  const int lane = threadIdx.x & 63;
  // everything that depends only on the row is the same in all lanes: said explicitly, so that it
  // lives in scalar registers and the branches on it are plain branches, not lane masks
  const int row = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (row >= rows) return;
  int s, h, i, nb;
  decode_row(meta, row, s, h, i, nb);
  const int64_t begin = sel_ptr[row];
  int n = __builtin_amdgcn_readfirstlane(int(sel_ptr[row + 1] - begin));
  n = min(n, i + 1);                            // never more than the causal-visible blocks
  if (n <= 0) return;
  int32_t* out = sel_idx + begin;
  if (lane == 0) {
    out[0] = 0;
    if (n >= 2) out[n - 1] = i;
  }
  const int want = n - 2;                       // picks among candidates 1..i-1
  if (want <= 0) return;
  const float* srow = scores + meta.score_off[s] + (int64_t(h) * nb + i) * nb;
  const int slots = (i + 63) >> 6;              // slots that hold at least one candidate
  if (slots <= 2) select_row<2>(srow, out, i, want, lane);
  else if (slots <= 4) select_row<4>(srow, out, i, want, lane);
  else if (slots <= 8) select_row<8>(srow, out, i, want, lane);
  else if (MAX_SLOTS <= 16 || slots <= 16) select_row<16>(srow, out, i, want, lane);
  else if (slots <= 32) select_row<(MAX_SLOTS > 16 ? 32 : 16)>(srow, out, i, want, lane);
  else select_row<MAX_SLOTS>(srow, out, i, want, lane);
}

}  // namespace

int32_t launch_select(const Geometry& g, const float* scores, const int64_t* sel_ptr,
                      int32_t* sel_idx, hipStream_t stream) {
  const int32_t rows = int32_t(g.rows);
  const dim3 grid((rows + 3) / 4), block(256);
  if (g.max_nb <= 1024)
    hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, stream, g.meta, scores, sel_ptr, sel_idx, rows);
  else
    hipLaunchKernelGGL(select_kernel<64>, grid, block, 0, stream, g.meta, scores, sel_ptr, sel_idx, rows);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
