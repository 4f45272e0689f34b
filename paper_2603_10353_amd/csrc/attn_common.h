// Helpers shared by the attention kernels (gfx950): vector types, LDS tile layout,
// direct global->LDS copies, LDS transpose reads.
#pragma once
#include "shplb_internal.h"

namespace shplb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int kKeysPerTile = 64;
constexpr int kRowBytes = 256;                          // one key row (128 bf16) in LDS
constexpr int kTileBytes = kKeysPerTile * kRowBytes;    // 16 KB per K or V tile
constexpr float kRescaleSlack = 8.0f;   // log2 units a row maximum may grow before O, l are rescaled
constexpr float kRowSumLimit = 8192.0f; // = 32 * 2^slack: a lane's 32 probabilities of a tile can only sum
                                        // to more if one of them exceeds 2^slack

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, v);
}

// Chunk swizzle of row r (only r mod 16 matters): a bijection on the 16 chunk slots.
// The two low row bits move a chunk by 64 bytes, bit 2 by 32 bytes, bit 3 by 16 bytes.
// A transpose read of V serves 32 lanes per cycle: four consecutive key rows, 64 bytes
// of each; with this they fall on the four different 64-byte quarters of the 64 banks
// (SQ_LDS_BANK_CONFLICT reads zero; with rows only 32 bytes apart every such read took
// twice as long).  Sixteen consecutive K rows read by the lanes of one operand fetch
// cover all sixteen slots under any bijection.
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1); }

// LDS transpose read: inside every group of 16 lanes, lane L receives element L%4 of
// the four 8-byte pieces addressed by lanes L/4, L/4+4, L/4+8, L/4+12.
__device__ __forceinline__ s16x4 lds_read_tr16(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}

__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0f70); }   // vmcnt(0)

// One wave copies 64 x 16 bytes from global memory (uniform base + per-lane byte
// offset) to the 1 KB of LDS starting at lds_base: lane l's 16 bytes land at
// lds_base + 16*l.  Issued as inline assembly so that the compiler's wait-count
// pass does not serialise every later LDS read behind it; completion is awaited
// explicitly (wait_vmem_all + barrier) before the stage is read.
__device__ __forceinline__ void copy_g2l_16(const char* base, uint32_t lane_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_base), "v"(lane_off), "s"(base)
               : "memory", "m0");
}

// acc + lo + hi of a packed bf16 pair (v_dot2c_f32_bf16 against (1, 1)).
__device__ __forceinline__ float dot2_ones(uint32_t packed, float acc) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), ones, acc, false);
}

// Exchange with lane ^ 32 without going through LDS.  v_permlane32_swap exchanges the
// upper half of its first register with the lower half of its second; fed two copies
// of x it leaves {x of the lower lane, x of the upper lane} of the pair in every lane.
// (Written as assembly: the two results must be two distinct registers.  The leading
// s_nop covers the wait states the swap needs after a VALU write of its operands.)
__device__ __forceinline__ void pair_values(float x, float& lower, float& upper) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  lower = a;
  upper = b;
}
// The raw exchange: afterwards the upper half of a holds what the lower half of b held and vice versa.
__device__ __forceinline__ void swap_halves(uint32_t& a, uint32_t& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float pair_max(float x) {
  float a, b;
  pair_values(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float pair_sum(float x) {
  float a, b;
  pair_values(x, a, b);
  return a + b;
}

// Partial results of the pieces of split rows travel between workgroups of one launch, possibly
// on different dies, whose L2 caches are not coherent with each other.  They are therefore written
// and read with device-scope accesses (relaxed atomics of 8 bytes: stores that write through to the
// level all dies see, loads that do not trust a die-local copy) instead of plain accesses between
// device-wide fences: such a fence writes back and invalidates the whole L2 of the die, which costs
// every other workgroup there its cached K/V tiles (measured: launches of a few hundred pieces took
// three times as long).
__device__ __forceinline__ void slot_store(float* p, float a, float b) {
  const uint64_t w = uint64_t(__float_as_uint(a)) | uint64_t(__float_as_uint(b)) << 32;
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void slot_load(const float* p, float& a, float& b) {
  const uint64_t w = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  a = __uint_as_float(uint32_t(w));
  b = __uint_as_float(uint32_t(w >> 32));
}
// 16-byte device-scope load.  Issued as assembly (there is no 16-byte atomic load to ask the compiler
// for); the data is not valid before slot_wait() has been called on it.
__device__ __forceinline__ f32x4 slot_load16_issue(const float* p) {
  f32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
  return v;
}
// Wait for all outstanding loads; the values pass through so that no use can be scheduled above the wait.
__device__ __forceinline__ void slot_wait(f32x4& a, f32x4& b, f32x4& c, f32x4& d) {
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : : "memory");
}
__device__ __forceinline__ void slot_store1(float* p, float a) {
  __hip_atomic_store(reinterpret_cast<uint32_t*>(p), __float_as_uint(a), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float slot_load1(const float* p) {
  return __uint_as_float(__hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// Pieces of split rows.  A piece leaves in its slot (slot_store) the unnormalised output O_c, the sum
// l_c of its probabilities, both relative to a reference exponent m_c (p = 2^(s*scale*log2e - m_c)),
// and is then counted (count_piece); the piece of a row that is counted last has the row combined
// (merge_row).  Softmax over the union of the pieces (Eq. 1 over the selected keys) is, with
// m = max_c m_c and w_c = 2^(m_c - m),
//
//     out = sum_c w_c O_c / sum_c w_c l_c,      lse = (m + log2 sum_c w_c l_c) ln 2,
//
// summed in piece order from the slots (the last piece reads its own result back like the others),
// so the result depends neither on which piece finished last nor on slot numbers.
constexpr int kMaxPieces = kSplitMaxPieces;
constexpr int kDeferredMerges = 1024;   // rows a workgroup can owe a merge (it stops taking items when full)

// Called by every thread of the workgroup after the piece's slot stores were issued.  Every thread
// waits until its stores are done, the workgroup meets at a barrier, one thread counts the piece with
// a device-scope atomic.  Returns (to all threads) whether this piece completed its row.
__device__ __forceinline__ bool count_piece(const SplitBuffers& sb, int pieces, int split_index, int32_t* s_flag) {
  // item records come from the ordering kernels; a malformed one must not index out of bounds
  if (pieces < 2 || pieces > kMaxPieces || split_index < 0 || split_index > sb.slot_capacity / 2) return false;
  wait_vmem_all();
  __syncthreads();
  if (threadIdx.x == 0)
    *s_flag = int(__hip_atomic_fetch_add(sb.done + split_index, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(*s_flag) == pieces - 1;
}

// Combine the pieces of one row into the output.  Two passes, so that few dependent memory round
// trips remain: first one thread per query turns the pieces' (m_c, l_c) into weights
// w_c / sum w_c l_c in LDS, then every thread accumulates its 16 output chunks piece by piece, the 16
// loads of a piece in flight together.  Kept out of line and called when nothing of the attention
// loop is live any more: inside that loop it cost the loop its register allocation (59 spilled
// registers against 4).
//   out_row: output of the row's first query (head applied); lse_row: likewise, or null;
//   n_valid: valid queries of the row (ragged last block);
//   lds_w, lds_l: kMaxPieces * BQ floats of LDS each.
template <int BQ, int THREADS>
__device__ __attribute__((noinline)) void merge_row(const SplitBuffers& sb, int pieces, int first_slot,
                                                    uint16_t* out_row, int64_t q_stride_t, float* lse_row,
                                                    int n_valid, float* lds_w, float* lds_l) {
  if (pieces < 2 || pieces > kMaxPieces || first_slot < 0 || first_slot + pieces > sb.slot_capacity) return;
  __syncthreads();                                  // the LDS tables are free (an earlier merge is over)
  const float* part_o = sb.part_o + int64_t(first_slot) * kSlotFloatsO;
  const float* part_ml = sb.part_ml + int64_t(first_slot) * kSlotFloatsML;
  // pass 1: thread q < BQ: weights of the pieces for query q, already divided by the denominator
  if (threadIdx.x < BQ) {
    const int q_in = threadIdx.x;
#pragma unroll 4
    for (int c = 0; c < pieces; ++c) {              // independent loads, several in flight
      lds_w[c * BQ + q_in] = slot_load1(part_ml + c * kSlotFloatsML + q_in);
      lds_l[c * BQ + q_in] = slot_load1(part_ml + c * kSlotFloatsML + 128 + q_in);
    }
    float m = -INFINITY;
    for (int c = 0; c < pieces; ++c) m = fmaxf(m, lds_w[c * BQ + q_in]);
    float l = 0.0f;
    for (int c = 0; c < pieces; ++c) {
      const float m_c = lds_w[c * BQ + q_in];
      const float w = m_c == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(m_c - m);
      lds_w[c * BQ + q_in] = w;
      l += w * lds_l[c * BQ + q_in];
    }
    const float inv = 1.0f / l;
    for (int c = 0; c < pieces; ++c) lds_w[c * BQ + q_in] *= inv;
    if (lse_row != nullptr && q_in < n_valid) lse_row[q_in] = (m + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
  }
  __syncthreads();
  // pass 2: the slots hold O in the order the attention kernels keep it in registers (slot_chunk()):
  // chunk e = ((wave * 4 + dt) * 4 + rq) * 64 + lane is dims 32 dt + 8 rq + 4 (lane / 32) .. +3 of query
  // 32 wave + lane % 32.  A thread owns chunks threadIdx.x + THREADS * u; a wave reads 1 KB runs.
  constexpr int kChunks = BQ * (kHeadDim / 4) / THREADS;
  static_assert(kChunks % 4 == 0, "chunks are awaited four at a time");
  f32x4 acc[kChunks];
#pragma unroll
  for (int u = 0; u < kChunks; ++u) acc[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  for (int c = 0; c < pieces; ++c) {
    f32x4 o[kChunks];
#pragma unroll
    for (int u = 0; u < kChunks; ++u)
      o[u] = slot_load16_issue(part_o + c * kSlotFloatsO + 4 * (threadIdx.x + THREADS * u));
#pragma unroll
    for (int u = 0; u < kChunks; u += 4) slot_wait(o[u], o[u + 1], o[u + 2], o[u + 3]);
#pragma unroll
    for (int u = 0; u < kChunks; ++u) {
      const int e = threadIdx.x + THREADS * u;
      const float w = lds_w[c * BQ + 32 * (e >> 10) + (e & 31)];
      acc[u] += w * o[u];
    }
  }
#pragma unroll
  for (int u = 0; u < kChunks; ++u) {
    const int e = threadIdx.x + THREADS * u;
    const int q_in = 32 * (e >> 10) + (e & 31);
    const int d = 32 * ((e >> 8) & 3) + 8 * ((e >> 6) & 3) + 4 * ((e >> 5) & 1);
    if (q_in >= n_valid) continue;                  // padding of a ragged last block
    u32x2 w2;
    w2.x = pack_bf16(acc[u].x, acc[u].y);
    w2.y = pack_bf16(acc[u].z, acc[u].w);
    *reinterpret_cast<u32x2*>(out_row + int64_t(q_in) * q_stride_t + d) = w2;
  }
}

// Where lane `lane` of wave `wave` keeps its four accumulator values rq of dim tile dt in a slot: the
// 64 lanes of a wave write one run of 1 KB (full cache lines, which write-through stores need).
__device__ __forceinline__ int slot_chunk(int wave, int dt, int rq, int lane) {
  return 4 * ((((wave * 4 + dt) * 4 + rq) << 6) + lane);
}

__device__ __forceinline__ uint32_t lds_offset_of(const void* p) {
  return uint32_t(size_t((__attribute__((address_space(3))) const char*)(p)));
}

}  // namespace shplb
