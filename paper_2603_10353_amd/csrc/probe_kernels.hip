// What the matrix pipe sustains on this chip, measured: a loop of nothing but
// v_mfma_f32_32x32x16_bf16 on register operands, eight waves per compute unit, no memory
// traffic.  With operands that look like the attention kernel's (random signs and mantissas,
// magnitudes around one) the chip holds a much lower clock than with constant operands, and
// that rate, not the nominal peak, is what a bf16 attention kernel can approach.  Used by the
// benchmark to put the measured ceiling next to its roofline figure.
#include "attn_common.h"

namespace shplb {
namespace {

template <int RANDOM>
__global__ __launch_bounds__(512) void mfma_rate_kernel(float* sink, uint64_t* clocks, int iters, uint32_t seed) {
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
  // eight operand sets per lane, cycled so that consecutive MFMAs never see the same pair
  u32x4 av[8], bv[8];
  uint32_t x = seed ^ (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
  auto bf16_bits = [](uint32_t r) {       // random sign, exponent 2^-2 .. 2^1, random mantissa; or one small constant
    return RANDOM ? (((r & 1u) << 15) | ((0x7du + ((r >> 1) & 3u)) << 7) | ((r >> 3) & 0x7fu)) : 0x3a83u;
  };
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      x = x * 1664525u + 1013904223u;
      const uint32_t r0 = x >> 8;
      x = x * 1664525u + 1013904223u;
      const uint32_t r1 = x >> 8;
      av[s][c] = bf16_bits(r0) | (bf16_bits(r0 >> 11) << 16);
      bv[s][c] = bf16_bits(r1) | (bf16_bits(r1 >> 11) << 16);
    }
  const uint64_t c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
      acc[s & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[s]),
                                                           __builtin_bit_cast(bf16x8, bv[(s + it) & 7]), acc[s & 3], 0, 0, 0);
  }
  const uint64_t c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  float total = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) total += acc[j][r];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = total;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = c1 - c0;                  // shader clock cycles of the loop
    clocks[1] = w1 - w0;                  // the same span in 100 MHz ticks
  }
}

}  // namespace

int32_t launch_mfma_rate(int random_operands, int iters, int n_workgroups, void* scratch, hipStream_t stream) {
  uint64_t* clocks = static_cast<uint64_t*>(scratch);
  float* sink = reinterpret_cast<float*>(clocks + 2);
  if (random_operands)
    hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(n_workgroups), dim3(512), 0, stream, sink, clocks, iters, 12345u);
  else
    hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(n_workgroups), dim3(512), 0, stream, sink, clocks, iters, 12345u);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
