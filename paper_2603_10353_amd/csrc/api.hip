// C-ABI entry points of libshplb: argument validation, geometry, workspace layout,
// the host-side greedy partition, and dispatch to the kernel launchers.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <mutex>
#include <numeric>
#include <vector>

#include "shplb_internal.h"

namespace shplb {

static inline int64_t align256(int64_t x) { return (x + 255) & ~int64_t(255); }

int32_t make_geometry(const shplb_problem* p, Geometry* g) {
  if (!p || !p->cu_seqlens) return SHPLB_E_NULL;
  if (p->n_seq < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1) return SHPLB_E_SHAPE;
  if (p->n_seq > SHPLB_MAX_SEQ) return SHPLB_E_UNSUPPORTED;
  // (sequence, head) pairs index the z dimension of the scoring grid
  if (int64_t(p->n_seq) * p->n_q_heads > SHPLB_MAX_SEQ_HEADS) return SHPLB_E_UNSUPPORTED;
  if (p->kv_head_of == nullptr) {
    if (p->n_q_heads % p->n_kv_heads) return SHPLB_E_SHAPE;
  } else {
    if (p->n_q_heads > SHPLB_MAX_MAPPED_HEADS || p->n_kv_heads > SHPLB_MAX_MAPPED_HEADS) return SHPLB_E_UNSUPPORTED;
    for (int h = 0; h < p->n_q_heads; ++h)
      if (p->kv_head_of[h] < 0 || p->kv_head_of[h] >= p->n_kv_heads) return SHPLB_E_SHAPE;
  }
  if (p->head_dim != kHeadDim) return SHPLB_E_UNSUPPORTED;
  if (p->block != 64 && p->block != 128) return SHPLB_E_UNSUPPORTED;
  if (p->cu_seqlens[0] != 0) return SHPLB_E_SHAPE;
  if (!(p->softmax_scale >= 0.0f) || !std::isfinite(p->softmax_scale)) return SHPLB_E_SHAPE;
  // head rows must be 16-byte aligned and must not overlap
  if (p->q_stride_h < kHeadDim || p->kv_stride_h < kHeadDim) return SHPLB_E_SHAPE;
  if (p->q_stride_t < p->q_stride_h * p->n_q_heads) return SHPLB_E_SHAPE;
  if (p->kv_stride_t < p->kv_stride_h * p->n_kv_heads) return SHPLB_E_SHAPE;
  if ((p->q_stride_t | p->q_stride_h | p->kv_stride_t | p->kv_stride_h) & 7) return SHPLB_E_SHAPE;
  if (p->q_stride_t >= (int64_t(1) << 24) || p->kv_stride_t >= (int64_t(1) << 24)) return SHPLB_E_UNSUPPORTED;

  std::memset(g, 0, sizeof(*g));
  SeqMeta& m = g->meta;
  m.n_seq = p->n_seq;
  m.n_q_heads = p->n_q_heads;
  m.n_kv_heads = p->n_kv_heads;
  m.block = p->block;
  m.kv_map = p->kv_head_of != nullptr;
  for (int h = 0; m.kv_map && h < p->n_q_heads; ++h) m.kv_of[h >> 2] |= uint32_t(p->kv_head_of[h]) << (8 * (h & 3));
  int64_t score_off = 0;
  int32_t max_nb = 0;
  for (int s = 0; s < p->n_seq; ++s) {
    const int64_t len = int64_t(p->cu_seqlens[s + 1]) - p->cu_seqlens[s];
    if (len < 1) return SHPLB_E_SHAPE;
    const int64_t nb = (len + p->block - 1) / p->block;
    if (nb > SHPLB_MAX_BLOCKS) return SHPLB_E_UNSUPPORTED;
    m.tok_begin[s] = p->cu_seqlens[s];
    m.blk_begin[s + 1] = m.blk_begin[s] + int32_t(nb);
    m.score_off[s] = score_off;
    score_off += int64_t(p->n_q_heads) * nb * nb;
    max_nb = std::max<int32_t>(max_nb, int32_t(nb));
  }
  m.tok_begin[p->n_seq] = p->cu_seqlens[p->n_seq];
  m.score_off[p->n_seq] = score_off;
  g->total_tokens = p->cu_seqlens[p->n_seq];
  g->total_blocks = m.blk_begin[p->n_seq];
  g->rows = g->total_blocks * p->n_q_heads;
  if (g->rows > (int64_t(1) << 30)) return SHPLB_E_UNSUPPORTED;
  g->max_nb = max_nb;
  g->st = Strides{p->q_stride_t, p->q_stride_h, p->kv_stride_t, p->kv_stride_h};
  g->scale = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / std::sqrt(float(kHeadDim));
  return SHPLB_OK;
}

WorkspaceLayout make_layout(const Geometry& g, int32_t split_slots, bool with_pooled) {
  WorkspaceLayout w;
  int64_t off = 0;
  w.qbar = off; off += with_pooled ? align256(int64_t(g.meta.n_q_heads) * g.total_blocks * kHeadDim * 6) : 0;
  w.kbar = off; off += with_pooled ? align256(int64_t(g.meta.n_kv_heads) * g.total_blocks * kHeadDim * 6) : 0;
  w.order_by_cost = off; off += align256(g.rows * 4);
  // Items: one per row plus the extra pieces of split rows.  split_length() keeps the pieces
  // within whatever number of slots it is given.
  w.slot_capacity = std::max<int32_t>(split_slots, 0);
  w.item_capacity = g.rows + w.slot_capacity;
  w.items = off; off += align256(w.item_capacity * int64_t(sizeof(ItemRec)));
  w.split_done = off; off += align256((w.slot_capacity / 2 + 1) * int64_t(sizeof(uint32_t)));
  w.split_count = off; off += 256;
  w.part_o = off; off += align256(w.slot_capacity * kSlotFloatsO * 4);
  w.part_ml = off; off += align256(w.slot_capacity * kSlotFloatsML * 4);
  const int64_t n_chunks = (g.rows + kOrderChunk - 1) / kOrderChunk;
  w.hist = off; off += align256(n_chunks * kCostBins * 4);
  w.bin_start = off; off += align256(int64_t(kCostBins) * 4);
  w.xcd_hist = off; off += align256(n_chunks * kXcds * 4);
  w.queue_begin = off; off += 256;
  w.tickets = off; off += align256(int64_t(kXcds) * kTicketStride * 4);
  w.total = off;
  return w;
}

int32_t persistent_workgroups(int block) {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return SHPLB_E_HIP;
  if (dev < 0 || dev >= 64) return SHPLB_E_HIP;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
      return SHPLB_E_HIP;
    cached[dev] = cus;
  }
  // two waves per SIMD: two 4-wave workgroups (128-token blocks) or four 2-wave ones (64) per compute unit
  return cached[dev] * (block == 64 ? 4 : 2);
}

}  // namespace shplb

using namespace shplb;

// Scratch of the entry point that allocates nothing (shplb_sparse_attn_prefill_static): the
// ordering kernels' histograms, the work-item queues and their tickets live here instead of in
// a caller's workspace.  The array's name is only a host-side handle; its device address is
// asked for once per device (every device holds its own copy) and that pointer is what the
// kernels get.
static __device__ __align__(256) unsigned char scratch[SHPLB_STATIC_SCRATCH_BYTES];

namespace {

std::mutex g_scratch_mutex;
void* g_scratch_ptr[64] = {nullptr};

// Device address of `scratch` on the current device.
int32_t static_scratch(void** ptr_out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SHPLB_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return SHPLB_E_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *ptr_out = g_scratch_ptr[dev];
  return SHPLB_OK;
}

}  // namespace

extern "C" {

int32_t shplb_num_rows(const shplb_problem* p, int64_t* rows_out) {
  if (!rows_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  *rows_out = g.rows;
  return SHPLB_OK;
}

int32_t shplb_max_blocks(const shplb_problem* p, int32_t* max_nb_out) {
  if (!max_nb_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  *max_nb_out = g.max_nb;
  return SHPLB_OK;
}

int32_t shplb_workspace_bytes(const shplb_problem* p, int64_t* bytes_out) {
  if (!bytes_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  *bytes_out = make_layout(g).total;
  return SHPLB_OK;
}

int32_t shplb_score_layout(const shplb_problem* p, int64_t* seq_offsets_out) {
  if (!seq_offsets_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  for (int s = 0; s <= g.meta.n_seq; ++s) seq_offsets_out[s] = g.meta.score_off[s];
  return SHPLB_OK;
}

int32_t shplb_sel_row_ptr(const shplb_problem* p, const int32_t* budgets, int64_t* sel_ptr_out) {
  if (!budgets || !sel_ptr_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  const SeqMeta& m = g.meta;
  for (int64_t x = 0; x < int64_t(m.n_seq) * m.n_q_heads; ++x)
    if (budgets[x] < 0) return SHPLB_E_BUDGET;
  int64_t row = 0, acc = 0;
  sel_ptr_out[0] = 0;
  for (int s = 0; s < m.n_seq; ++s) {
    const int64_t nb = m.blk_begin[s + 1] - m.blk_begin[s];
    for (int h = 0; h < m.n_q_heads; ++h) {
      const int64_t keep = std::min<int64_t>(std::max<int64_t>(budgets[s * m.n_q_heads + h], 2), nb);
      for (int64_t i = 0; i < nb; ++i) {
        acc += std::min<int64_t>(keep, i + 1);
        sel_ptr_out[++row] = acc;
      }
    }
  }
  return SHPLB_OK;
}

int32_t shplb_sched_num_workgroups(const shplb_problem* p, int32_t* n_out) {
  if (!n_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  const int32_t n = persistent_workgroups(g.meta.block);
  if (n < 0) return n;
  *n_out = n;
  return SHPLB_OK;
}

int32_t shplb_block_scores(const shplb_problem* p, const void* q, const void* k,
                           float* scores_out, void* workspace, void* stream) {
  if (!q || !k || !scores_out || !workspace) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k)) & 15) return SHPLB_E_SHAPE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return SHPLB_E_SHAPE;
  const WorkspaceLayout w = make_layout(g);
  char* ws = static_cast<char*>(workspace);
  const int32_t n_wg = persistent_workgroups();   // two per compute unit
  if (n_wg < 0) return SHPLB_E_HIP;
  return launch_pool_scores(g, q, k, scores_out, reinterpret_cast<uint16_t*>(ws + w.qbar),
                            reinterpret_cast<uint16_t*>(ws + w.kbar), n_wg / 2, static_cast<hipStream_t>(stream));
}

int32_t shplb_select_topk_per_head(const shplb_problem* p, const float* scores,
                                   const int32_t* budgets, const int64_t* sel_ptr,
                                   int32_t* sel_idx_out, void* stream) {
  if (!scores || !budgets || !sel_ptr || !sel_idx_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  for (int64_t x = 0; x < int64_t(g.meta.n_seq) * g.meta.n_q_heads; ++x)
    if (budgets[x] < 0) return SHPLB_E_BUDGET;
  return launch_select(g, scores, sel_ptr, sel_idx_out, static_cast<hipStream_t>(stream));
}

namespace {

int32_t attention_entry(const shplb_problem* p, const void* q, const void* k, const void* v,
                        const int64_t* sel_ptr, const int32_t* sel_idx, void* out, float* lse_out,
                        void* sched_stats_out, void* workspace, int32_t split_slots, void* stream,
                        bool static_scratch_call = false) {
  if (!q || !k || !v || !sel_ptr || !sel_idx || !out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  if (static_scratch_call) {
    // the attention step's part of the workspace only (no pooled planes), inside the static array
    if (make_layout(g, 0, false).total > SHPLB_STATIC_SCRATCH_BYTES) return SHPLB_E_WORKSPACE;
    if (int32_t st = static_scratch(&workspace)) return st;
  }
  if (!workspace) return SHPLB_E_NULL;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) |
       reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(out)) & 15)
    return SHPLB_E_SHAPE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return SHPLB_E_SHAPE;
  const int32_t n_wg = persistent_workgroups(g.meta.block);
  if (n_wg < 0) return n_wg;
  const WorkspaceLayout w = make_layout(g, split_slots, !static_scratch_call);
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (int32_t rc = launch_order(g, sel_ptr, w, ws, n_wg, st)) return rc;
  const WorkQueues wq{reinterpret_cast<const ItemRec*>(ws + w.items),
                      reinterpret_cast<const int32_t*>(ws + w.queue_begin),
                      reinterpret_cast<uint32_t*>(ws + w.tickets)};
  const SplitBuffers sb{reinterpret_cast<float*>(ws + w.part_o), reinterpret_cast<float*>(ws + w.part_ml),
                        reinterpret_cast<uint32_t*>(ws + w.split_done),
                        reinterpret_cast<SplitCounters*>(ws + w.split_count), int32_t(w.slot_capacity)};
  return launch_attention(g, q, k, v, sel_ptr, sel_idx, out, lse_out, static_cast<shplb_wg_stats*>(sched_stats_out),
                          wq, sb, n_wg, st);
}

}  // namespace

int32_t shplb_sparse_attn_prefill(const shplb_problem* p, const void* q, const void* k,
                                  const void* v, const int64_t* sel_ptr, const int32_t* sel_idx,
                                  void* out, float* lse_out, void* sched_stats_out,
                                  void* workspace, void* stream) {
  return attention_entry(p, q, k, v, sel_ptr, sel_idx, out, lse_out, sched_stats_out, workspace, 0, stream);
}

int32_t shplb_sparse_attn_prefill_static(const shplb_problem* p, const void* q, const void* k,
                                         const void* v, const int64_t* sel_ptr, const int32_t* sel_idx,
                                         void* out, float* lse_out, void* sched_stats_out, void* stream) {
  return attention_entry(p, q, k, v, sel_ptr, sel_idx, out, lse_out, sched_stats_out, nullptr, 0, stream, true);
}

int32_t shplb_split_workspace_bytes(const shplb_problem* p, int32_t split_slots, int64_t* bytes_out) {
  if (!bytes_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  if (split_slots < 2 || split_slots > kSplitSlotsMax) return SHPLB_E_UNSUPPORTED;
  *bytes_out = make_layout(g, split_slots).total;
  return SHPLB_OK;
}

int32_t shplb_sparse_attn_prefill_split(const shplb_problem* p, const void* q, const void* k,
                                        const void* v, const int64_t* sel_ptr, const int32_t* sel_idx,
                                        void* out, float* lse_out, void* sched_stats_out,
                                        void* workspace, int32_t split_slots, void* stream) {
  if (!p) return SHPLB_E_NULL;
  if (split_slots < 2 || split_slots > kSplitSlotsMax) return SHPLB_E_UNSUPPORTED;
  return attention_entry(p, q, k, v, sel_ptr, sel_idx, out, lse_out, sched_stats_out, workspace, split_slots,
                         stream);
}

// Offline recovery profile of Section 2.4 at block granularity: a dense causal pass.
int32_t shplb_block_mass(const shplb_problem* p, const void* q, const void* k, float* mass_out, void* stream) {
  if (!q || !k || !mass_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k)) & 15) return SHPLB_E_SHAPE;
  return launch_block_mass(g, q, k, mass_out, static_cast<hipStream_t>(stream));
}

// Offline recovery ratio of Section 2.4 at token granularity: the top-k weights of every query.
int32_t shplb_token_recovery(const shplb_problem* p, const void* q, const void* k, const int32_t* budgets,
                             int32_t n_budgets, float* recovery_out, void* stream) {
  if (!q || !k || !recovery_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k)) & 15) return SHPLB_E_SHAPE;
  if (n_budgets < 1 || n_budgets > SHPLB_MAX_TOKEN_BUDGETS) return SHPLB_E_UNSUPPORTED;
  if (!budgets) return SHPLB_E_NULL;
  for (int b = 0; b < n_budgets; ++b)
    if (budgets[b] < 1) return SHPLB_E_BUDGET;
  return launch_token_recovery(g, q, k, budgets, n_budgets, recovery_out, static_cast<hipStream_t>(stream));
}

int32_t shplb_token_recovery_heads(const shplb_problem* p, const float* recovery, int32_t n_budgets,
                                   double* heads_out) {
  if (!recovery || !heads_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  if (n_budgets < 1 || n_budgets > SHPLB_MAX_TOKEN_BUDGETS) return SHPLB_E_UNSUPPORTED;
  const int64_t tokens = g.total_tokens;
  for (int h = 0; h < g.meta.n_q_heads; ++h)
    for (int b = 0; b < n_budgets; ++b) {
      const float* src = recovery + (int64_t(b) * g.meta.n_q_heads + h) * tokens;
      double sum = 0.0;
      for (int64_t t = 0; t < tokens; ++t) sum += src[t];
      heads_out[int64_t(h) * n_budgets + b] = sum / double(tokens);
    }
  return SHPLB_OK;
}

int32_t shplb_recovery_curves(const shplb_problem* p, const float* mass, int32_t n_levels, double* curves_out) {
  if (!mass || !curves_out) return SHPLB_E_NULL;
  Geometry g;
  if (int32_t st = make_geometry(p, &g)) return st;
  if (n_levels != g.max_nb + 1) return SHPLB_E_SHAPE;
  const SeqMeta& m = g.meta;
  const int n_heads = m.n_q_heads;
  std::fill(curves_out, curves_out + int64_t(n_heads) * n_levels, 0.0);
  std::vector<double> row;
  for (int s = 0; s < m.n_seq; ++s) {
    const int nb = m.blk_begin[s + 1] - m.blk_begin[s];
    const int len = m.tok_begin[s + 1] - m.tok_begin[s];
    for (int h = 0; h < n_heads; ++h)
      for (int i = 0; i < nb; ++i) {
        const int n_valid = std::min(m.block, len - i * m.block);
        const float* src = mass + m.score_off[s] + (int64_t(h) * nb + i) * nb;
        row.assign(src, src + i + 1);
        std::sort(row.begin(), row.end(), std::greater<double>());        // heaviest first
        double* dst = curves_out + int64_t(h) * n_levels;
        double cum = 0.0;
        for (int b = 1; b < n_levels; ++b) {
          if (b <= i + 1) cum += row[b - 1];
          dst[b] += n_valid * cum;
        }
      }
  }
  for (int64_t x = 0; x < int64_t(n_heads) * n_levels; ++x) curves_out[x] /= double(g.total_tokens);
  return SHPLB_OK;
}

// Greedy multiway partition of Section 3.3.  n is a head (or KV-group) count, so
// the O(n * n_parts) scan for the least-loaded part is as good as a heap here.
int32_t shplb_balance_heads(const int64_t* costs, int32_t n, int32_t n_parts,
                            int32_t max_per_part, int32_t* part_of_out, int64_t* loads_out) {
  if (n < 0 || n_parts < 1 || max_per_part < 0) return SHPLB_E_SHAPE;
  if (n > 0 && (!costs || !part_of_out)) return SHPLB_E_NULL;
  if (max_per_part > 0 && int64_t(max_per_part) * n_parts < n) return SHPLB_E_BUDGET;
  for (int32_t x = 0; x < n; ++x)
    if (costs[x] < 0) return SHPLB_E_BUDGET;
  std::vector<int32_t> visit(n);
  std::iota(visit.begin(), visit.end(), 0);
  std::stable_sort(visit.begin(), visit.end(),
                   [&](int32_t a, int32_t b) { return costs[a] > costs[b]; });
  std::vector<int64_t> load(n_parts, 0);
  std::vector<int32_t> held(n_parts, 0);
  for (int32_t x : visit) {
    int32_t to = -1;
    for (int32_t d = 0; d < n_parts; ++d) {
      if (max_per_part > 0 && held[d] >= max_per_part) continue;
      if (to < 0 || load[d] < load[to]) to = d;
    }
    part_of_out[x] = to;
    load[to] += costs[x];
    held[to] += 1;
  }
  if (loads_out) std::copy(load.begin(), load.end(), loads_out);
  return SHPLB_OK;
}

int32_t shplb_shift_budgets(const double* recovery, int32_t n_heads, int32_t n_levels,
                            int64_t total, int32_t lower, int32_t step,
                            int32_t* budgets_out, int64_t* n_moves_out) {
  if (n_heads < 1 || n_levels < 1 || step < 1 || lower < 0) return SHPLB_E_SHAPE;
  if (!recovery || !budgets_out) return SHPLB_E_NULL;
  auto rec = [&](int32_t h, int64_t b) { return recovery[int64_t(h) * n_levels + b]; };
  for (int32_t h = 0; h < n_heads; ++h)
    for (int32_t b = 0; b < n_levels; ++b) {
      if (!std::isfinite(rec(h, b))) return SHPLB_E_SHAPE;
      if (b > 0 && rec(h, b) < rec(h, b - 1)) return SHPLB_E_SHAPE;
    }
  if (total < 0) return SHPLB_E_BUDGET;
  std::vector<int64_t> b(n_heads);
  for (int32_t h = 0; h < n_heads; ++h) b[h] = total / n_heads + (h < total % n_heads ? 1 : 0);
  if (b[n_heads - 1] < lower || b[0] > n_levels - 1) return SHPLB_E_BUDGET;
  int64_t moves = 0;
  std::vector<double> now(n_heads);
  for (;;) {
    for (int32_t h = 0; h < n_heads; ++h) now[h] = rec(h, b[h]);
    int32_t recv = 0;
    for (int32_t h = 1; h < n_heads; ++h)
      if (now[h] < now[recv]) recv = h;
    int32_t give = -1;
    for (int32_t h = 0; h < n_heads; ++h)
      if (h != recv && b[h] - step >= lower && (give < 0 || now[h] > now[give])) give = h;
    if (give < 0 || b[recv] + step > n_levels - 1) break;            // nothing left to move
    const double give_after = rec(give, b[give] - step), recv_after = rec(recv, b[recv] + step);
    double min_after = std::min(give_after, recv_after);
    for (int32_t h = 0; h < n_heads; ++h)
      if (h != give && h != recv) min_after = std::min(min_after, now[h]);
    if (min_after < now[recv]) break;                                 // the move would not help
    b[give] -= step;
    b[recv] += step;
    moves += 1;
    if (give_after <= min_after) break;                               // the giver is the new minimum
  }
  for (int32_t h = 0; h < n_heads; ++h) budgets_out[h] = int32_t(b[h]);
  if (n_moves_out) *n_moves_out = moves;
  return SHPLB_OK;
}

int32_t shplb_probe_mfma_rate(int32_t random_operands, int32_t iters, int32_t n_workgroups, void* scratch,
                              void* stream) {
  if (!scratch) return SHPLB_E_NULL;
  if (iters < 1 || n_workgroups < 1 || (reinterpret_cast<uintptr_t>(scratch) & 7)) return SHPLB_E_SHAPE;
  return launch_mfma_rate(random_operands, iters, n_workgroups, scratch, static_cast<hipStream_t>(stream));
}

const char* shplb_strerror(int32_t status) {
  switch (status) {
    case SHPLB_OK: return "ok";
    case SHPLB_E_NULL: return "required pointer is null";
    case SHPLB_E_SHAPE: return "bad shape, stride, alignment, scale or cu_seqlens";
    case SHPLB_E_BUDGET: return "negative budget or cost, or partition cannot hold the units";
    case SHPLB_E_WORKSPACE: return "problem needs more scratch than the static array holds";
    case SHPLB_E_UNSUPPORTED: return "unsupported configuration (head_dim 128, block 64/128, <=64 sequences, <=4096 blocks each)";
    case SHPLB_E_HIP: return "HIP call or kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
