// Internal declarations shared by the translation units of libshplb (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "shplb.h"

namespace shplb {

constexpr int kHeadDim = 128;
constexpr int kCostBins = 4100;       // selected-block counts 0..SHPLB_MAX_BLOCKS, rounded up
constexpr int kOrderChunk = 256;      // rows per workgroup in the ordering kernels
constexpr int kXcds = 8;              // accelerator dies (XCDs) of an MI355X, each with its own L2
constexpr int kTicketStride = 16;     // uint32 slots between two queue tickets (one 64-byte line each)
constexpr int kSplitSlotsMax = 1 << 16;   // most partial-result slots a caller may ask for (64 KB + 1 KB each)
constexpr int kSplitMinTiles = 32;    // a piece of a split row covers at least this many 64-key tiles: a piece costs
                                      // about 7 us more than it computes for (write-through stores of its partial
                                      // result, the count) and a merge 12-15 us; 32 tiles are about 50 us of work
constexpr int kSplitShare = 2;        // rows longer than 1/kSplitShare of a workgroup's average share are split
constexpr int64_t kSlotFloatsO = 128 * kHeadDim;   // one partial result: unnormalised O of up to 128 queries ...
constexpr int64_t kSlotFloatsML = 2 * 128;         // ... and their reference exponent and denominator

// Sequence geometry, passed to kernels by value (about 1 KB of kernel arguments).
struct SeqMeta {
  int32_t n_seq;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t block;
  int32_t tok_begin[SHPLB_MAX_SEQ + 1];   // cu_seqlens
  int32_t blk_begin[SHPLB_MAX_SEQ + 1];   // cumulative block counts
  int64_t score_off[SHPLB_MAX_SEQ + 1];   // float offset of each sequence's score cube
  int32_t kv_map;                         // 1: kv_of[] holds the KV head of every query head
  uint32_t kv_of[SHPLB_MAX_MAPPED_HEADS / 4];   // one byte per query head, four to a word
};

struct Strides {
  int64_t q_t, q_h, kv_t, kv_h;
};

// Validated, host-side view of a shplb_problem.
struct Geometry {
  SeqMeta meta;
  Strides st;
  int64_t total_tokens;
  int64_t total_blocks;
  int64_t rows;
  int32_t max_nb;
  float scale;
};

// Workspace carve-up (byte offsets, each 256-byte aligned).
struct WorkspaceLayout {
  int64_t qbar, kbar;        // pooled blocks as three bf16 planes, each [H][total_blocks][128]
  int64_t order_by_cost;     // int32 [rows]: rows by descending cost (intermediate)
  int64_t items;             // ItemRec [item_capacity]: the work items, one queue per XCD after the other
  int64_t split_done;        // uint32 [slot_capacity / 2 + 1]: pieces finished, per split row
  int64_t split_count;       // SplitCounters
  int64_t part_o;            // float [slot_capacity][128][kHeadDim]: partial results of the pieces
  int64_t part_ml;           // float [slot_capacity][2][128]
  int64_t item_capacity, slot_capacity;   // counts, not offsets
  int64_t hist;              // int32 [n_chunks][kCostBins]
  int64_t bin_start;         // int32 [kCostBins]
  int64_t xcd_hist;          // int32 [n_chunks][kXcds]
  int64_t queue_begin;       // int32 [kXcds + 1]: queue x is items[queue_begin[x] .. queue_begin[x+1])
  int64_t tickets;           // uint32 [kXcds * kTicketStride]
  int64_t total;
};

int32_t make_geometry(const shplb_problem* p, Geometry* g);
// split_slots: partial-result slots for rows split along the keys (0: rows stay whole)
// with_pooled = false leaves out the pooled planes (the attention step alone does not use them)
WorkspaceLayout make_layout(const Geometry& g, int32_t split_slots = 0, bool with_pooled = true);
// Persistent workgroups of an attention launch on the current device: as many as fit at two waves
// per SIMD (two per compute unit with 128-token blocks, four with 64); <0 on HIP error.
int32_t persistent_workgroups(int block = 128);

// Kernel launchers (each returns a SHPLB status).
int32_t launch_pool_scores(const Geometry& g, const void* q, const void* k, float* scores,
                           uint16_t* q_planes, uint16_t* k_planes, int n_compute_units, hipStream_t stream);
int32_t launch_select(const Geometry& g, const float* scores, const int64_t* sel_ptr,
                      int32_t* sel_idx, hipStream_t stream);
int32_t launch_order(const Geometry& g, const int64_t* sel_ptr, const WorkspaceLayout& w,
                     char* workspace, int32_t n_wg, hipStream_t stream);
int32_t launch_mfma_rate(int random_operands, int iters, int n_workgroups, void* scratch, hipStream_t stream);
int32_t launch_block_mass(const Geometry& g, const void* q, const void* k, float* mass, hipStream_t stream);
int32_t launch_token_recovery(const Geometry& g, const void* q, const void* k, const int32_t* budgets,
                              int32_t n_budgets, float* recovery, hipStream_t stream);
// One work item of an attention launch: a row, or one piece of a row that was split along
// its selected key blocks (positions [first, first + n_sel) of the row's selection).
struct alignas(32) ItemRec {
  int32_t row;
  int32_t n_sel;        // selected key blocks this item covers
  int64_t sel_begin;    // index of its first one in sel_idx
  int32_t slot;         // partial-result slot it writes, or -1: the item is the whole row and writes the output
  int32_t pieces;       // pieces of its row (1: whole row)
  int32_t first_slot;   // slot of the row's first piece; the row's pieces hold slots first_slot .. + pieces - 1
  int32_t split_index;  // the row's entry in the finished-pieces counters
};

struct SplitCounters {
  uint32_t n_slots, n_rows;   // slots handed out, rows split (zeroed by the ordering kernels)
};

// Longest item, in key blocks, of a launch whose rows select total_cost blocks in all, run by
// n_wg persistent workgroups, with room for slot_capacity partial results (0: never split).
// Rows longer than this are cut into near-equal pieces, so that no single item is a large
// part of a workgroup's average share (total / n_wg) and a launch of few rows still fills the
// chip.  Three lower bounds: a piece covers at least kSplitMinTiles key tiles (an item's fixed
// cost must stay small beside its work); no longer than needed (1/kSplitShare of the share:
// at long contexts nothing is split); and the pieces must fit the slots: a split row of n
// blocks has ceil(n / len) < 2 n / len pieces, so all split rows together have fewer than
// 2 total / len <= slot_capacity.
__host__ __device__ inline int64_t split_length(int64_t total_cost, int slot_capacity, int n_wg, int block) {
  if (slot_capacity < 2) return int64_t(1) << 40;
  int64_t len = kSplitMinTiles * 64 / block;
  const int64_t fit = (2 * total_cost + slot_capacity - 1) / slot_capacity;
  const int64_t share = (total_cost + int64_t(n_wg) * kSplitShare - 1) / (int64_t(n_wg) * kSplitShare);
  if (fit > len) len = fit;
  if (share > len) len = share;
  return len;
}
constexpr int kSplitMaxPieces = 64;   // pieces of one row (their weights meet in a fixed piece of LDS)
__host__ __device__ inline int pieces_of(int64_t n_sel, int64_t split_len) {
  if (n_sel <= split_len) return 1;
  const int64_t p = (n_sel + split_len - 1) / split_len;
  return int(p < kSplitMaxPieces ? p : kSplitMaxPieces);
}
// piece c of a row of n selected blocks cut into p pieces covers [piece_begin(c), piece_begin(c + 1))
__host__ __device__ inline int64_t piece_begin(int64_t n_sel, int p, int c) { return n_sel * c / p; }

// The per-XCD work queues the ordering kernels build (device pointers into the workspace).
struct WorkQueues {
  const ItemRec* items;        // items, queue after queue, each by descending row cost
  const int32_t* queue_begin;  // [kXcds + 1]
  uint32_t* tickets;           // [kXcds * kTicketStride], zeroed by the ordering kernels
};

// Where the pieces of split rows leave their results, and the per-row counts of finished pieces.
struct SplitBuffers {
  float* part_o;
  float* part_ml;
  uint32_t* done;              // [slot_capacity / 2 + 1], zeroed by the ordering kernels
  SplitCounters* count;
  int32_t slot_capacity;
};

int32_t launch_attention(const Geometry& g, const void* q, const void* k, const void* v,
                         const int64_t* sel_ptr, const int32_t* sel_idx, void* out, float* lse,
                         shplb_wg_stats* stats, WorkQueues wq, SplitBuffers sb, int32_t n_wg, hipStream_t stream);

// KV head that query head h reads: the caller's map, or equal groups of consecutive heads.
__device__ __forceinline__ int kv_head_of(const SeqMeta& m, int h) {
  return m.kv_map ? int(m.kv_of[h >> 2] >> (8 * (h & 3)) & 0xff) : h / (m.n_q_heads / m.n_kv_heads);
}

// Row -> (sequence, head, query block).  Rows of one sequence are contiguous.
__device__ __forceinline__ void decode_row(const SeqMeta& m, int32_t row, int& s, int& h, int& i, int& nb) {
  s = 0;
  while (s + 1 < m.n_seq && row >= m.blk_begin[s + 1] * m.n_q_heads) ++s;
  const int local = row - m.blk_begin[s] * m.n_q_heads;
  nb = m.blk_begin[s + 1] - m.blk_begin[s];
  h = local / nb;
  i = local - h * nb;
}

// Home XCD of a row.  All rows that stream the same K/V (one KV head of one sequence) go to
// the same die, so its L2 sees one K/V stream per resident head instead of all of them;
// with fewer streams than dies a stream is spread over several dies by query block.
__device__ __forceinline__ int xcd_of_row(const SeqMeta& m, int32_t row) {
  int s, h, i, nb;
  decode_row(m, row, s, h, i, nb);
  const int stream = s * m.n_kv_heads + kv_head_of(m, h);
  const int n_streams = m.n_seq * m.n_kv_heads;
  if (n_streams >= kXcds) return stream % kXcds;
  const int per = kXcds / n_streams;
  return stream * per + i % per;
}

// The queue with the most items left, other than those in empty_mask (ties: the first one
// after home), or -1.  Counts are read with device-scope loads and may be a little old.
// Kept out of line: it runs a few times per workgroup, at the end of a launch, and inlined
// it costs the attention kernels registers across their whole item loop.
__device__ __attribute__((noinline)) int fullest_queue(const int32_t* queue_begin, const uint32_t* tickets,
                                                       int home, int empty_mask) {
  int most = 0, pick = -1;
  for (int d = 1; d < kXcds; ++d) {
    const int x = (home + d) % kXcds;
    if (empty_mask & 1 << x) continue;
    const uint32_t size = uint32_t(queue_begin[x + 1] - queue_begin[x]);
    const uint32_t taken = __hip_atomic_load(tickets + x * kTicketStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int left = taken < size ? int(size - taken) : 0;
    if (left > most) {
      most = left;
      pick = x;
    }
  }
  return pick;
}

// Next work item for a persistent workgroup (called by one thread).  A workgroup draws from
// its home die's queue until that is empty; from then on every item comes from the queue
// that has the most items left at that moment.  Helpers so spread over the dies that still
// have work in proportion to what is left there, and no queue is left for last with its
// heavy items still in it.  An old count only affects which queue is tried, the ticket
// decides.  A queue whose ticket came back past its end is never tried again, so the loop
// ends after at most kXcds misses.  Returns the item's position in wq.items, or -1 when
// every queue is empty.
__device__ __forceinline__ int32_t next_item(const WorkQueues& wq, int home, int& empty_mask) {
  int pick = home;
  for (;;) {
    if (empty_mask & 1 << home) {
      pick = fullest_queue(wq.queue_begin, wq.tickets, home, empty_mask);
      if (pick < 0) return -1;
    }
    const int begin = wq.queue_begin[pick], end = wq.queue_begin[pick + 1];
    const uint32_t t = atomicAdd(wq.tickets + pick * kTicketStride, 1u);
    if (t < uint32_t(end - begin)) return begin + int(t);
    empty_mask |= 1 << pick;
  }
}

__device__ __forceinline__ int my_xcd() {
  return int(__builtin_amdgcn_s_getreg((4 - 1) << 11 | 0 << 6 | 20) & 0xf) % kXcds;   // XCC_ID[3:0]
}

}  // namespace shplb
