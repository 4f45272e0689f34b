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
// the same K/V blocks sit next to each other in a queue.
//
// When the caller provides slots for partial results (shplb_sparse_attn_prefill_split), rows
// longer than split_length() are cut along their selected key blocks into near-equal pieces,
// each an item of its own (the pieces of a row sit next to each other, where the row would).
// A piece leaves a partial result in a slot of the workspace; the piece of a row that finishes
// last combines them (count_piece() and merge_row() in attn_common.h).  Slots and counter entries are handed
// out through atomic counters, so their numbering varies between runs; what is computed does
// not depend on it.
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
// earlier chunks + rows of the same bin earlier in this chunk.  Counts the row's pieces into
// the die histogram of the chunk its position falls in (sort 2, pass 1).
__global__ __launch_bounds__(kOrderChunk) void order_scatter_kernel(
    SeqMeta meta, const int64_t* __restrict__ sel_ptr, const int32_t* __restrict__ hist,
    const int32_t* __restrict__ bin_start, int32_t* __restrict__ order_by_cost,
    int32_t* __restrict__ xcd_hist, int rows, int n_bins, int slot_capacity, int n_wg) {
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
  const int64_t split_len = split_length(sel_ptr[rows] - sel_ptr[0], slot_capacity, n_wg, meta.block);
  const int pieces = pieces_of(sel_ptr[row + 1] - sel_ptr[row], split_len);
  atomicAdd(&xcd_hist[(pos / kOrderChunk) * kXcds + xcd_of_row(meta, row)], pieces);
}

// Sort 2, pass 2 (one workgroup of 8 waves, wave x scans die x): exclusive prefix of the
// die histogram over chunks, queue boundaries, fresh tickets and split counters.
__global__ __launch_bounds__(64 * kXcds) void queue_scan_kernel(
    int32_t* __restrict__ xcd_hist, int32_t* __restrict__ queue_begin, uint32_t* __restrict__ tickets,
    SplitCounters* __restrict__ split_count, int n_chunks) {
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
    split_count->n_slots = 0;
    split_count->n_rows = 0;
    int32_t run = 0;
    for (int d = 0; d < kXcds; ++d) {
      queue_begin[d] = run;
      run += total[d];
    }
    queue_begin[kXcds] = run;
  }
}

// The items of one row: the row itself, or its pieces (then with a run of slots and a counter
// of finished pieces).  Returns without writing if the slots or counters are exhausted, which
// split_length() rules out.
__device__ __forceinline__ void write_items(ItemRec* __restrict__ dst, int row, int64_t sel_begin, int64_t n_sel,
                                            int pieces, uint32_t* __restrict__ split_done,
                                            SplitCounters* __restrict__ split_count, int slot_capacity) {
  if (pieces <= 1) {                     // a whole row: no 64-bit divisions for piece boundaries
    ItemRec rec;
    rec.row = row;
    rec.n_sel = int32_t(max(n_sel, int64_t(0)));
    rec.sel_begin = sel_begin;
    rec.slot = -1;
    rec.pieces = pieces;
    rec.first_slot = -1;
    rec.split_index = -1;
    dst[0] = rec;
    return;
  }
  int slot = -1, entry = -1;
  if (pieces > 1) {
    slot = int(atomicAdd(&split_count->n_slots, uint32_t(pieces)));
    if (slot + pieces > slot_capacity) return;
    entry = int(atomicAdd(&split_count->n_rows, 1u));
    if (entry >= slot_capacity / 2 + 1) return;
    split_done[entry] = 0;
  }
  for (int c = 0; c < pieces; ++c) {
    const int64_t first = piece_begin(n_sel, pieces, c);
    ItemRec rec;
    rec.row = row;
    rec.n_sel = int32_t(max(piece_begin(n_sel, pieces, c + 1) - first, int64_t(0)));
    rec.sel_begin = sel_begin + first;
    rec.slot = pieces > 1 ? slot + c : -1;
    rec.pieces = pieces;
    rec.first_slot = slot;
    rec.split_index = entry;
    dst[c] = rec;
  }
}

// Sort 2, pass 3: write the items of the cost-sorted rows into their die's queue.  A row's
// place is the number of pieces of earlier rows of the same die.
__global__ __launch_bounds__(kOrderChunk) void queue_scatter_kernel(
    SeqMeta meta, const int64_t* __restrict__ sel_ptr, const int32_t* __restrict__ order_by_cost,
    const int32_t* __restrict__ xcd_hist, const int32_t* __restrict__ queue_begin, ItemRec* __restrict__ items,
    uint32_t* __restrict__ split_done, SplitCounters* __restrict__ split_count, int rows, int item_capacity,
    int slot_capacity, int n_wg) {
  __shared__ int32_t die[kOrderChunk];
  __shared__ int32_t n_pieces[kOrderChunk];
  const int pos = blockIdx.x * kOrderChunk + threadIdx.x;
  const int row = pos < rows ? order_by_cost[pos] : -1;
  const int x = row >= 0 ? xcd_of_row(meta, row) : -1;
  const int64_t split_len = split_length(sel_ptr[rows] - sel_ptr[0], slot_capacity, n_wg, meta.block);
  const int64_t sel_begin = row >= 0 ? sel_ptr[row] : 0;
  const int64_t n_sel = row >= 0 ? sel_ptr[row + 1] - sel_begin : 0;
  const int pieces = pieces_of(n_sel, split_len);
  die[threadIdx.x] = x;
  n_pieces[threadIdx.x] = pieces;
  __syncthreads();
  if (row < 0) return;
  int before = 0;
  for (int t = 0; t < int(threadIdx.x); ++t) before += die[t] == x ? n_pieces[t] : 0;
  const int dst = queue_begin[x] + xcd_hist[blockIdx.x * kXcds + x] + before;
  if (dst < 0 || dst + pieces > item_capacity) return;   // never taken (see split_length); keeps stores in bounds
  write_items(items + dst, row, sel_begin, n_sel, pieces, split_done, split_count, slot_capacity);
}

// Both sorts in one workgroup, for launches of few rows (prompts of a few thousand tokens, a
// part's share of a layer), where five dependent launches would cost more than the sorting.
// One counting sort over the combined key (die, descending cost) with the histogram in LDS:
// count, scan, place; a row counts as many items as it has pieces.  Rows of equal key are
// placed in the order their atomics arrive, so unlike the two-sort path the order among equal
// costs is not fixed; it decides only which workgroup takes which of two equally long rows.
constexpr int kSmallThreads = 1024;
constexpr int kSmallKeys = 16384;     // LDS histogram entries: kXcds * (cost bins) must fit
constexpr int kSmallRows = 16384;

__global__ __launch_bounds__(kSmallThreads) void order_small_kernel(
    SeqMeta meta, const int64_t* __restrict__ sel_ptr, ItemRec* __restrict__ items,
    int32_t* __restrict__ queue_begin, uint32_t* __restrict__ tickets, uint32_t* __restrict__ split_done,
    SplitCounters* __restrict__ split_count, int rows, int n_bins, int item_capacity, int slot_capacity,
    int n_wg) {
  __shared__ int32_t slot[kSmallKeys];               // count per key, then next free position per key
  __shared__ int32_t wave_sum[kSmallThreads / 64];
  const int tid = threadIdx.x;
  const int n_keys = kXcds * n_bins;
  for (int x = tid; x < n_keys; x += kSmallThreads) slot[x] = 0;
  if (tid < kXcds) tickets[tid * kTicketStride] = 0;
  if (tid == 0) {
    split_count->n_slots = 0;
    split_count->n_rows = 0;
  }
  __syncthreads();                                   // also orders the counters' reset before their use below
  const int64_t split_len = split_length(sel_ptr[rows] - sel_ptr[0], slot_capacity, n_wg, meta.block);
  auto key_of = [&](int row) {
    return xcd_of_row(meta, row) * n_bins + (n_bins - 1 - min(cost_bin(sel_ptr, row), n_bins - 1));
  };
  auto pieces_of_row = [&](int row) { return pieces_of(sel_ptr[row + 1] - sel_ptr[row], split_len); };
  for (int row = tid; row < rows; row += kSmallThreads) atomicAdd(&slot[key_of(row)], pieces_of_row(row));
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
  if (tid == kSmallThreads - 1) queue_begin[kXcds] = run;    // the last thread's run ends at the item count
  __syncthreads();
  for (int row = tid; row < rows; row += kSmallThreads) {
    const int64_t sel_begin = sel_ptr[row];
    const int64_t n_sel = max(sel_ptr[row + 1] - sel_begin, int64_t(0));
    const int pieces = pieces_of(n_sel, split_len);
    const int dst = atomicAdd(&slot[key_of(row)], pieces);
    if (dst < 0 || dst + pieces > item_capacity) continue;   // never taken (see split_length)
    write_items(items + dst, row, sel_begin, n_sel, pieces, split_done, split_count, slot_capacity);
  }
}

}  // namespace

int32_t launch_order(const Geometry& g, const int64_t* sel_ptr, const WorkspaceLayout& w,
                     char* workspace, int32_t n_wg, hipStream_t stream) {
  const int rows = int(g.rows);
  const int n_chunks = (rows + kOrderChunk - 1) / kOrderChunk;
  const int n_bins = min(g.max_nb + 1, kCostBins);
  int32_t* hist = reinterpret_cast<int32_t*>(workspace + w.hist);
  int32_t* bin_start = reinterpret_cast<int32_t*>(workspace + w.bin_start);
  int32_t* order_by_cost = reinterpret_cast<int32_t*>(workspace + w.order_by_cost);
  ItemRec* items = reinterpret_cast<ItemRec*>(workspace + w.items);
  uint32_t* split_done = reinterpret_cast<uint32_t*>(workspace + w.split_done);
  SplitCounters* split_count = reinterpret_cast<SplitCounters*>(workspace + w.split_count);
  int32_t* xcd_hist = reinterpret_cast<int32_t*>(workspace + w.xcd_hist);
  int32_t* queue_begin = reinterpret_cast<int32_t*>(workspace + w.queue_begin);
  uint32_t* tickets = reinterpret_cast<uint32_t*>(workspace + w.tickets);
  if (rows <= kSmallRows && kXcds * n_bins <= kSmallKeys) {
    hipLaunchKernelGGL(order_small_kernel, dim3(1), dim3(kSmallThreads), 0, stream, g.meta, sel_ptr, items,
                       queue_begin, tickets, split_done, split_count, rows, n_bins, int(w.item_capacity),
                       int(w.slot_capacity), n_wg);
    if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
    return SHPLB_OK;
  }
  hipLaunchKernelGGL(order_hist_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, sel_ptr, hist, xcd_hist,
                     rows, n_bins);
  hipLaunchKernelGGL(order_scan_kernel, dim3(1), dim3(1024), 0, stream, hist, bin_start, n_chunks, n_bins);
  hipLaunchKernelGGL(order_scatter_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, g.meta, sel_ptr, hist,
                     bin_start, order_by_cost, xcd_hist, rows, n_bins, int(w.slot_capacity), n_wg);
  hipLaunchKernelGGL(queue_scan_kernel, dim3(1), dim3(64 * kXcds), 0, stream, xcd_hist, queue_begin, tickets,
                     split_count, n_chunks);
  hipLaunchKernelGGL(queue_scatter_kernel, dim3(n_chunks), dim3(kOrderChunk), 0, stream, g.meta, sel_ptr,
                     order_by_cost, xcd_hist, queue_begin, items, split_done, split_count, rows,
                     int(w.item_capacity), int(w.slot_capacity), n_wg);
  if (hipGetLastError() != hipSuccess) return SHPLB_E_HIP;
  return SHPLB_OK;
}

}  // namespace shplb
