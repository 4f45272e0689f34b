// Work-item ordering for the persistent attention launch.
//
// The paper's greedy (Section 3.3) sorts units by descending cost and hands each to the
// least-loaded worker.  On one GPU the workers are compute units: the rows (sequence,
// head, query block) are sorted by descending selected-block count and consumed through
// atomic tickets, so the next-largest item always goes to a workgroup that just became
// free.  MI355X has eight dies (XCDs), each with its own L2, so the sorted list is split
// into one queue per die: all rows that stream one KV head of one sequence share a home
// die, whose L2 then sees that K/V once.  A workgroup drains its die's queue first and
// then helps whichever die has the most items left (see next_item()), which keeps the
// greedy's balance when the dies' queues hold very different amounts of work.
//
// Two stable counting sorts, least significant key first:
//   1. by descending cost (per-256-row histograms, one-workgroup scan, scatter);
//   2. by home die (8 bins; its histogram is accumulated by the first scatter).
// Equal keys keep their row order (head-major, then query block), so items that stream
// the same K/V blocks sit next to each other in a queue.  Everything is deterministic.
#include "shplb_internal.h"

namespace shplb {
namespace {

__device__ __forceinline__ int cost_bin(const int64_t* sel_ptr, int row) {
  const int64_t c = sel_ptr[row + 1] - sel_ptr[row];
  return int(c < 0 ? 0 : (c > kCostBins - 1 ? kCostBins - 1 : c));
}

// Sort 1, pass 1: per-chunk histogram of costs, hist[chunk][bin]; also clears the die
// histogram of the chunk for sort 2.
__global__ __launch_bounds__(kOrderChunk) void order_hist_kernel(
    const int64_t* __restrict__ sel_ptr, int32_t* __restrict__ hist, int32_t* __restrict__ xcd_hist,
    int rows, int n_bins) {
  __shared__ int32_t h[kCostBins];
  for (int b = threadIdx.x; b < n_bins; b += kOrderChunk) h[b] = 0;
  if (threadIdx.x < kXcds) xcd_hist[blockIdx.x * kXcds + threadIdx.x] = 0;
  __syncthreads();
  const int row = blockIdx.x * kOrderChunk + threadIdx.x;
  if (row < rows) atomicAdd(&h[min(cost_bin(sel_ptr, row), n_bins - 1)], 1);
  __syncthreads();
  int32_t* dst = hist + int64_t(blockIdx.x) * n_bins;
  for (int b = threadIdx.x; b < n_bins; b += kOrderChunk) dst[b] = h[b];
}

// Sort 1, pass 2 (one workgroup): turn hist[chunk][bin] into the exclusive count of
// earlier chunks within the bin, and bin_start[bin] into the number of rows in costlier
// bins.
__global__ __launch_bounds__(1024) void order_scan_kernel(
    int32_t* __restrict__ hist, int32_t* __restrict__ bin_start, int n_chunks, int n_bins) {
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
}

// Sort 1, pass 3: scatter.  Position = rows in costlier bins + rows of the same bin in
// earlier chunks + rows of the same bin earlier in this chunk.  Counts the row into the
// die histogram of the chunk its position falls in (sort 2, pass 1).
__global__ __launch_bounds__(kOrderChunk) void order_scatter_kernel(
    SeqMeta meta, const int64_t* __restrict__ sel_ptr, const int32_t* __restrict__ hist,
    const int32_t* __restrict__ bin_start, int32_t* __restrict__ order_by_cost,
    int32_t* __restrict__ xcd_hist, int rows, int n_bins) {
  __shared__ int32_t bins[kOrderChunk];
  const int row = blockIdx.x * kOrderChunk + threadIdx.x;
  const int bin = row < rows ? min(cost_bin(sel_ptr, row), n_bins - 1) : -1;
  bins[threadIdx.x] = bin;
  __syncthreads();
  if (row >= rows) return;
  int rank = 0;
  for (int x = 0; x < int(threadIdx.x); ++x) rank += bins[x] == bin;
  const int pos = bin_start[bin] + hist[int64_t(blockIdx.x) * n_bins + bin] + rank;
  order_by_cost[pos] = row;
  atomicAdd(&xcd_hist[(pos / kOrderChunk) * kXcds + xcd_of_row(meta, row)], 1);
}

// Sort 2, pass 2 (one workgroup of 8 waves, wave x scans die x): exclusive prefix of the
// die histogram over chunks, queue boundaries, and fresh tickets.
__global__ __launch_bounds__(64 * kXcds) void queue_scan_kernel(
    int32_t* __restrict__ xcd_hist, int32_t* __restrict__ queue_begin, uint32_t* __restrict__ tickets,
    int n_chunks) {
  __shared__ int32_t total[kXcds];
  const int x = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int32_t carry = 0;
  for (int base = 0; base < n_chunks; base += 64) {
    const int c = base + lane;
    const int32_t v = c < n_chunks ? xcd_hist[c * kXcds + x] : 0;
    int32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int32_t up = __shfl_up(inc, d);
      if (lane >= d) inc += up;
    }
    if (c < n_chunks) xcd_hist[c * kXcds + x] = carry + inc - v;
    carry += __shfl(inc, 63);
  }
  if (lane == 0) {
    total[x] = carry;
    tickets[x * kTicketStride] = 0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int32_t run = 0;
    for (int d = 0; d < kXcds; ++d) {
      queue_begin[d] = run;
      run += total[d];
    }
    queue_begin[kXcds] = run;
  }
}

// Sort 2, pass 3: scatter the cost-sorted rows into their die's queue.
__global__ __launch_bounds__(kOrderChunk) void queue_scatter_kernel(
    SeqMeta meta, const int32_t* __restrict__ order_by_cost, const int32_t* __restrict__ xcd_hist,
    const int32_t* __restrict__ queue_begin, int32_t* __restrict__ order, int rows) {
  __shared__ int32_t die[kOrderChunk];
  const int pos = blockIdx.x * kOrderChunk + threadIdx.x;
  const int row = pos < rows ? order_by_cost[pos] : -1;
  const int x = row >= 0 ? xcd_of_row(meta, row) : -1;
  die[threadIdx.x] = x;
  __syncthreads();
  if (row < 0) return;
  int rank = 0;
  for (int t = 0; t < int(threadIdx.x); ++t) rank += die[t] == x;
  order[queue_begin[x] + xcd_hist[blockIdx.x * kXcds + x] + rank] = row;
}

// Both sorts in one workgroup, for launches of few rows (prompts of a few thousand tokens, a
// part's share of a layer), where five dependent launches would cost more than the sorting.
// One counting sort over the combined key (die, descending cost) with the histogram in LDS:
// count, scan, place.  Rows of equal key are placed in the order their atomics arrive, so
// unlike the two-sort path the order among equal costs is not fixed; it decides only which
// workgroup takes which of two equally long rows.
constexpr int kSmallThreads = 1024;
constexpr int kSmallKeys = 16384;     // LDS histogram entries: kXcds * (cost bins) must fit
constexpr int kSmallRows = 16384;

__global__ __launch_bounds__(kSmallThreads) void order_small_kernel(
    SeqMeta meta, const int64_t* __restrict__ sel_ptr, int32_t* __restrict__ order,
    int32_t* __restrict__ queue_begin, uint32_t* __restrict__ tickets, int rows, int n_bins) {
  __shared__ int32_t slot[kSmallKeys];               // count per key, then next free position per key
  __shared__ int32_t wave_sum[kSmallThreads / 64];
  const int tid = threadIdx.x;
  const int n_keys = kXcds * n_bins;
  for (int x = tid; x < n_keys; x += kSmallThreads) slot[x] = 0;
  if (tid < kXcds) tickets[tid * kTicketStride] = 0;
  __syncthreads();
  auto key_of = [&](int row) {
    return xcd_of_row(meta, row) * n_bins + (n_bins - 1 - min(cost_bin(sel_ptr, row), n_bins - 1));
  };
  for (int row = tid; row < rows; row += kSmallThreads) atomicAdd(&slot[key_of(row)], 1);
  __syncthreads();
  // exclusive scan over the keys: a thread owns a run of consecutive keys
  const int per = (n_keys + kSmallThreads - 1) / kSmallThreads;
  const int k0 = min(tid * per, n_keys), k1 = min(k0 + per, n_keys);
  int32_t mine = 0;
  for (int x = k0; x < k1; ++x) mine += slot[x];
  int32_t inc = mine;                                // inclusive scan of the threads' sums inside the wave
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int32_t up = __shfl_up(inc, d);
    if ((tid & 63) >= d) inc += up;
  }
  if ((tid & 63) == 63) wave_sum[tid >> 6] = inc;
  __syncthreads();
  int32_t run = inc - mine;
  for (int w = 0; w < (tid >> 6); ++w) run += wave_sum[w];
  for (int x = k0; x < k1; ++x) {
    const int32_t c = slot[x];
    slot[x] = run;
    if (x % n_bins == 0) queue_begin[x / n_bins] = run;   // first key of a die: its queue starts here
    run += c;
  }
  if (tid == 0) queue_begin[kXcds] = rows;
  __syncthreads();
  for (int row = tid; row < rows; row += kSmallThreads) order[atomicAdd(&slot[key_of(row)], 1)] = row;
}

}  // namespace

int32_t launch_order(const Geometry& g, const int64_t* sel_ptr, const WorkspaceLayout& w,
                     char* workspace, hipStream_t stream) {
  const int rows = int(g.rows);
  const int n_chunks = (rows + kOrderChunk - 1) / kOrderChunk;
  const int n_bins = min(g.max_nb + 1, kCostBins);
  int32_t* hist = reinterpret_cast<int32_t*>(workspace + w.hist);
  int32_t* bin_start = reinterpret_cast<int32_t*>(workspace + w.bin_start);
  int32_t* order_by_cost = reinterpret_cast<int32_t*>(workspace + w.order_by_cost);
  int32_t* order = reinterpret_cast<int32_t*>(workspace + w.order);
  int32_t* xcd_hist = reinterpret_cast<int32_t*>(workspace + w.xcd_hist);
  int32_t* queue_begin = reinterpret_cast<int32_t*>(workspace + w.queue_begin);
  uint32_t* tickets = reinterpret_cast<uint32_t*>(workspace + w.tickets);
  if (rows <= kSmallRows && kXcds * n_bins <= kSmallKeys) {
    hipLaunchKernelGGL(order_small_kernel, dim3(1), dim3(kSmallThreads), 0, stream, g.meta, sel_ptr, order,
                       queue_begin, tickets, rows, n_bins);
    if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
    return SHPLB_OK;
  }
  hipLaunchKernelGGL(order_hist_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, sel_ptr, hist, xcd_hist,
                     rows, n_bins);
  hipLaunchKernelGGL(order_scan_kernel, dim3(1), dim3(1024), 0, stream, hist, bin_start, n_chunks, n_bins);
  hipLaunchKernelGGL(order_scatter_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, g.meta, sel_ptr, hist,
                     bin_start, order_by_cost, xcd_hist, rows, n_bins);
  hipLaunchKernelGGL(queue_scan_kernel, dim3(1), dim3(64 * kXcds), 0, stream, xcd_hist, queue_begin, tickets,
                     n_chunks);
  hipLaunchKernelGGL(queue_scatter_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, g.meta, order_by_cost,
                     xcd_hist, queue_begin, order, rows);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
