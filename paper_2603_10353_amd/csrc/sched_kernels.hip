// Work-item ordering for the persistent attention launch: a stable counting sort of
// the (sequence, head, query block) rows by descending selected-block count.
//
// The paper's greedy (Section 3.3) sorts units by descending cost and hands each to
// the least-loaded worker.  On one GPU the workers are compute units: the sorted
// list built here is consumed through a single atomic ticket, so the next-largest
// item always goes to whichever workgroup becomes free first.
// Equal costs keep their row order (head-major, then query block), which keeps
// items that stream the same K/V blocks next to each other in time.
#include "shplb_internal.h"

namespace shplb {
namespace {

__device__ __forceinline__ int cost_bin(const int64_t* sel_ptr, int row) {
  const int64_t c = sel_ptr[row + 1] - sel_ptr[row];
  return int(c < 0 ? 0 : (c > kCostBins - 1 ? kCostBins - 1 : c));
}

// Pass 1: per-chunk histogram of costs.  hist[chunk][bin].
__global__ __launch_bounds__(kOrderChunk) void order_hist_kernel(
    const int64_t* __restrict__ sel_ptr, int32_t* __restrict__ hist, int rows, int n_bins) {
  __shared__ int32_t h[kCostBins];
  for (int b = threadIdx.x; b < n_bins; b += kOrderChunk) h[b] = 0;
  __syncthreads();
  const int row = blockIdx.x * kOrderChunk + threadIdx.x;
  if (row < rows) atomicAdd(&h[min(cost_bin(sel_ptr, row), n_bins - 1)], 1);
  __syncthreads();
  int32_t* dst = hist + int64_t(blockIdx.x) * n_bins;
  for (int b = threadIdx.x; b < n_bins; b += kOrderChunk) dst[b] = h[b];
}

// Pass 2 (one workgroup): turn hist[chunk][bin] into the exclusive count of earlier
// chunks within the bin, and bin_start[bin] into the number of rows in costlier
// bins.  Also resets the ticket the attention kernel draws from.
__global__ __launch_bounds__(1024) void order_scan_kernel(
    int32_t* __restrict__ hist, int32_t* __restrict__ bin_start, uint32_t* __restrict__ ticket,
    int n_chunks, int n_bins) {
  __shared__ int32_t total[kCostBins];
  __shared__ int32_t wave_sum[16];
  for (int b = threadIdx.x; b < n_bins; b += 1024) {
    int32_t run = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += 8) {      // loads of a batch are independent
      int32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = c0 + u < n_chunks ? hist[int64_t(c0 + u) * n_bins + b] : 0;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u < n_chunks) hist[int64_t(c0 + u) * n_bins + b] = run;
        run += v[u];
      }
    }
    total[b] = run;
  }
  __syncthreads();
  // exclusive scan of totals in descending-cost order: position x <-> bin n_bins-1-x
  int32_t carry = 0;
  for (int base = 0; base < n_bins; base += 1024) {
    const int x = base + threadIdx.x;
    const int32_t v = x < n_bins ? total[n_bins - 1 - x] : 0;
    int32_t inc = v;                               // inclusive scan inside the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int32_t up = __shfl_up(inc, d);
      if ((threadIdx.x & 63) >= d) inc += up;
    }
    if ((threadIdx.x & 63) == 63) wave_sum[threadIdx.x >> 6] = inc;
    __syncthreads();
    int32_t before = carry;
    for (int w = 0; w < int(threadIdx.x >> 6); ++w) before += wave_sum[w];
    if (x < n_bins) bin_start[n_bins - 1 - x] = before + inc - v;
    int32_t all = 0;
    for (int w = 0; w < 16; ++w) all += wave_sum[w];
    carry += all;
    __syncthreads();
  }
  if (threadIdx.x == 0) ticket[0] = 0;
}

// Pass 3: scatter.  Position = rows in costlier bins + rows of the same bin in
// earlier chunks + rows of the same bin earlier in this chunk.
__global__ __launch_bounds__(kOrderChunk) void order_scatter_kernel(
    const int64_t* __restrict__ sel_ptr, const int32_t* __restrict__ hist,
    const int32_t* __restrict__ bin_start, int32_t* __restrict__ order, int rows, int n_bins) {
  __shared__ int32_t bins[kOrderChunk];
  const int row = blockIdx.x * kOrderChunk + threadIdx.x;
  const int bin = row < rows ? min(cost_bin(sel_ptr, row), n_bins - 1) : -1;
  bins[threadIdx.x] = bin;
  __syncthreads();
  if (row >= rows) return;
  int rank = 0;
  for (int x = 0; x < int(threadIdx.x); ++x) rank += bins[x] == bin;
  order[bin_start[bin] + hist[int64_t(blockIdx.x) * n_bins + bin] + rank] = row;
}

}  // namespace

int32_t launch_order(const Geometry& g, const int64_t* sel_ptr, const WorkspaceLayout& w,
                     char* workspace, hipStream_t stream) {
  const int rows = int(g.rows);
  const int n_chunks = (rows + kOrderChunk - 1) / kOrderChunk;
  const int n_bins = min(g.max_nb + 1, kCostBins);
  int32_t* hist = reinterpret_cast<int32_t*>(workspace + w.hist);
  int32_t* bin_start = reinterpret_cast<int32_t*>(workspace + w.bin_start);
  int32_t* order = reinterpret_cast<int32_t*>(workspace + w.order);
  uint32_t* ticket = reinterpret_cast<uint32_t*>(workspace + w.ticket);
  hipLaunchKernelGGL(order_hist_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, sel_ptr, hist, rows, n_bins);
  hipLaunchKernelGGL(order_scan_kernel, dim3(1), dim3(1024), 0, stream, hist, bin_start, ticket, n_chunks, n_bins);
  hipLaunchKernelGGL(order_scatter_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, sel_ptr, hist,
                     bin_start, order, rows, n_bins);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
