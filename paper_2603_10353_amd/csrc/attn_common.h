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

__device__ __forceinline__ uint32_t lds_offset_of(const void* p) {
  return uint32_t(size_t((__attribute__((address_space(3))) const char*)(p)));
}

}  // namespace shplb
