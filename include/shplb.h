/*
 * shplb.h -- C ABI of the S-HPLB hot path on one MI355X (gfx950).
 *
 * The path: causal attention prefill in which every head runs under its own
 * sparsity budget (paper Sections 3.1-3.3).  Three device steps and one host step:
 *
 *   shplb_block_scores          pooled query/key block importance logits
 *   shplb_select_topk_per_head  per-head top-k key-block selection
 *   shplb_sparse_attn_prefill   block-sparse causal attention over the selection,
 *                               work items dealt to compute units by descending cost
 *   shplb_balance_heads         greedy head-to-partition assignment (host)
 *   shplb_shift_budgets         max-min budget shifting: the producer of the budgets (host)
 *   shplb_block_mass            offline recovery profile: attention weight per block pair
 *   shplb_recovery_curves       recovery ratio per head and budget from that profile (host)
 *   shplb_token_recovery        offline recovery ratio at token granularity, per query
 *   shplb_token_recovery_heads  its mean per head (host)
 *
 * Conventions
 *   - Every function returns an int32 status: 0 = OK, negative = error (see
 *     SHPLB_E_*).  Nothing throws.  shplb_strerror() gives a text.
 *   - "device" pointers are HIP device memory owned by the caller; the library
 *     never allocates, frees or keeps them.  "host" pointers are ordinary memory,
 *     read (or written) synchronously before the call returns.
 *   - Device work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and is asynchronous; outputs are bit-identical from run
 *     to run (each work item owns its output rows; scheduling order never changes
 *     results).
 *   - Tensors are token-major: Q is [T, n_q_heads, head_dim] bf16 with element
 *     strides (q_stride_t, q_stride_h, 1); K and V are [T, n_kv_heads, head_dim]
 *     bf16 with strides (kv_stride_t, kv_stride_h, 1).  T = cu_seqlens[n_seq].
 *     Base pointers and strides must keep every head row 16-byte aligned.
 *   - Sequences are split into blocks of `block` tokens; a block never straddles
 *     two sequences; the last block of a sequence may be ragged.
 *     nb_s = ceil(len_s / block).
 *   - Row index of (sequence s, query head h, query block i):
 *       row = (sum_{s'<s} nb_s') * n_q_heads + h * nb_s + i.
 *   - GQA: query head h reads KV head h / (n_q_heads / n_kv_heads) (Section 2.1).
 *     A GPU's share under the head-to-device assignment of Section 3.3 is an
 *     arbitrary set of query heads, so its heads need not form whole groups of equal
 *     size: kv_head_of, when not NULL, gives the KV head (0 .. n_kv_heads-1, among
 *     the KV heads this call is given) of every query head, and n_q_heads need not
 *     be a multiple of n_kv_heads (both at most SHPLB_MAX_MAPPED_HEADS then).
 */
#ifndef SHPLB_H
#define SHPLB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SHPLB_API __attribute__((visibility("default")))

#define SHPLB_OK              0
#define SHPLB_E_NULL        (-1)  /* a required pointer is NULL */
#define SHPLB_E_SHAPE       (-2)  /* bad shape, stride, alignment or cu_seqlens */
#define SHPLB_E_BUDGET      (-3)  /* negative budget, or partition cannot hold the units */
#define SHPLB_E_WORKSPACE   (-4)  /* the problem needs more scratch than shplb_sparse_attn_prefill_static has */
#define SHPLB_E_UNSUPPORTED (-5)  /* head_dim != 128, block not 64/128, too many sequences/blocks/heads */
#define SHPLB_E_HIP         (-6)  /* a HIP call or kernel launch failed */

#define SHPLB_MAX_SEQ        64    /* sequences per call */
#define SHPLB_MAX_BLOCKS   4096    /* blocks per sequence */
#define SHPLB_MAX_SEQ_HEADS 65535  /* n_seq * n_q_heads per call */
#define SHPLB_MAX_MAPPED_HEADS 256  /* n_q_heads and n_kv_heads with an explicit kv_head_of */
#define SHPLB_MAX_TOKEN_BUDGETS 8  /* budgets per shplb_token_recovery call */

typedef struct {
  int32_t n_seq;                 /* 1..SHPLB_MAX_SEQ */
  const int32_t* cu_seqlens;     /* host [n_seq+1]; cu[0] = 0, strictly increasing */
  int32_t n_q_heads, n_kv_heads; /* n_q_heads % n_kv_heads == 0 unless kv_head_of is given */
  int32_t head_dim;              /* 128 */
  int32_t block;                 /* 64 or 128 */
  int64_t q_stride_t, q_stride_h;   /* element strides of Q (and of the output O) */
  int64_t kv_stride_t, kv_stride_h; /* element strides of K and V */
  float softmax_scale;           /* > 0, or 0 for 1/sqrt(head_dim) (Eq. 1) */
  const int32_t* kv_head_of;     /* host [n_q_heads], or NULL: see below */
} shplb_problem;

/* Per-workgroup record written by shplb_sparse_attn_prefill when asked for. */
typedef struct {
  uint32_t xcc_id;        /* accelerator die the workgroup ran on */
  uint32_t cu_id;         /* (shader engine << 8) | compute unit inside the die */
  uint32_t n_items;       /* (head, query block) items it processed */
  uint32_t cost_blocks;   /* selected key blocks over those items */
  uint64_t t_first;       /* constant-rate device clock at its first item */
  uint64_t t_last;        /* ... after its last item */
} shplb_wg_stats;

/* ---- host-side shape helpers (no device work) --------------------------- */

/* Number of (sequence, head, query block) rows. */
SHPLB_API int32_t shplb_num_rows(const shplb_problem* p, int64_t* rows_out /*host*/);

/* Largest block count of any sequence, max_s nb_s (shplb_recovery_curves takes
 * n_levels = this + 1). */
SHPLB_API int32_t shplb_max_blocks(const shplb_problem* p, int32_t* max_nb_out /*host*/);

/* Bytes of device workspace any entry point below needs for this problem. */
SHPLB_API int32_t shplb_workspace_bytes(const shplb_problem* p, int64_t* bytes_out /*host*/);

/* Layout of the score buffer: sequence s occupies floats
 * [seq_offsets[s], seq_offsets[s+1]) as a row-major [n_q_heads, nb_s, nb_s]
 * array; seq_offsets[n_seq] is the total float count. */
SHPLB_API int32_t shplb_score_layout(const shplb_problem* p, int64_t* seq_offsets_out /*host [n_seq+1]*/);

/* CSR row pointer of the selection, closed form: row (s,h,i) holds
 * min(clamp(budgets[s*n_q_heads+h], 2, nb_s), i+1) blocks -- the head's budget
 * (in blocks, applied to every query-block row of the head; Section 3.1), never
 * fewer than the always-kept sink and diagonal blocks, never more than the
 * causal-visible blocks. */
SHPLB_API int32_t shplb_sel_row_ptr(const shplb_problem* p, const int32_t* budgets /*host [n_seq*n_q_heads]*/,
                          int64_t* sel_ptr_out /*host [rows+1]*/);

/* Workgroups the attention launch uses on the current device (size of the
 * sched_stats_out array). */
SHPLB_API int32_t shplb_sched_num_workgroups(const shplb_problem* p, int32_t* n_out /*host*/);

/* ---- device steps -------------------------------------------------------- */

/* Block importance (the estimator the paper leaves to its borrowed kernels,
 * Section 4; scale from Eq. 1): mean-pool the valid tokens of every query block
 * and key block, then scores[s][h][i][j] = (Qbar[h,i] . Kbar[h/G,j]) * scale for
 * j <= i.  Entries with j > i are not written.  Means, products and sums carry
 * fp32 precision (products are formed from exact three-way bf16 splits of the
 * fp32 means and accumulated in fp32).
 *   q, k: device bf16.  scores_out: device fp32, shplb_score_layout() floats.
 *   workspace: device, shplb_workspace_bytes(). */
SHPLB_API int32_t shplb_block_scores(const shplb_problem* p, const void* q, const void* k,
                           float* scores_out, void* workspace, void* stream);

/* Per-head top-k selection (Sections 2.3-2.4: a per-head budget applied as a
 * top-k, which needs only the order of the scores).  Row (s,h,i) keeps block 0
 * and block i, then the highest-scoring blocks among 1..i-1 until it holds
 * sel_ptr[row+1]-sel_ptr[row] blocks; equal scores go to the lower block index
 * (+0 and -0 are equal; NaN scores are a caller error).  Indices are written
 * ascending.
 *   scores: device fp32 as written by shplb_block_scores.
 *   budgets: host [n_seq*n_q_heads], validated (>= 0); sel_ptr: device int64
 *   [rows+1], the array shplb_sel_row_ptr() fills for the same budgets.
 *   sel_idx_out: device int32 [sel_ptr[rows]]. */
SHPLB_API int32_t shplb_select_topk_per_head(const shplb_problem* p, const float* scores,
                                   const int32_t* budgets, const int64_t* sel_ptr,
                                   int32_t* sel_idx_out, void* stream);

/* Block-sparse causal attention (Eq. 1 restricted to the selected key blocks,
 * token-level causal mask inside the diagonal block), bf16 MFMA with fp32
 * accumulation and fp32 online softmax.  Work items are the rows; they are
 * ordered by descending selected-block count and handed to persistent
 * workgroups through one queue per accelerator die with an atomic ticket each:
 * the greedy rule of Section 3.3 (largest first, to whichever worker is free
 * first) applied to compute units.
 *   sel_ptr/sel_idx: device CSR; every row's list must be ascending, within
 *   [0, i], and contain i (lists written by shplb_select_topk_per_head are).
 *   out: device bf16 [T, n_q_heads, head_dim], strides as Q.
 *   lse_out: device fp32 [n_q_heads, T] natural-log softmax denominators, or NULL.
 *   sched_stats_out: device shplb_wg_stats[shplb_sched_num_workgroups()], or NULL.
 *   workspace: device, shplb_workspace_bytes(); must not be shared with a call
 *   still in flight on another stream. */
SHPLB_API int32_t shplb_sparse_attn_prefill(const shplb_problem* p, const void* q, const void* k,
                                  const void* v, const int64_t* sel_ptr, const int32_t* sel_idx,
                                  void* out, float* lse_out, void* sched_stats_out,
                                  void* workspace, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the attention step of
 * shplb_sparse_attn_prefill with its scratch (ordering histograms, work-item queues, tickets)
 * in a static device array of SHPLB_STATIC_SCRATCH_BYTES inside the library instead of a
 * workspace argument.  Same kernels, same results, bit for bit.  It allocates and frees
 * nothing.  The scratch needed is about 100 bytes per (sequence, head, query block) row: the
 * array covers about 80 000 rows (a 128K-token layer of 32 heads has 32 768); a larger
 * problem is refused with SHPLB_E_WORKSPACE before any device work.
 * Every GPU the library is used on holds its own copy of the array until the process ends.
 * All calls on one GPU share it: the kernels rewrite everything they read, so calls in
 * sequence on one stream need no clearing in between, but two calls that overlap on one GPU
 * (different streams, different threads) race and must not be made.  The first call on a
 * device looks up the array's address (hipGetSymbolAddress): make it once outside any
 * stream capture.
 *   Arguments as for shplb_sparse_attn_prefill, without the workspace. */
#define SHPLB_STATIC_SCRATCH_BYTES (8 << 20)
SHPLB_API int32_t shplb_sparse_attn_prefill_static(const shplb_problem* p, const void* q, const void* k,
                                         const void* v, const int64_t* sel_ptr, const int32_t* sel_idx,
                                         void* out, float* lse_out, void* sched_stats_out, void* stream);

/* The same attention step with long rows cut along their selected key blocks
 * (the partition of Section 3.3 applied below the row: a work item is a row or a
 * piece of one).  A row is cut into near-equal pieces (at most 64) when it selects
 * more blocks than L = max(2048 keys, ceil(total / (2 * workgroups)), ceil(2 *
 * total / split_slots)), total = all selected blocks of the call: rows that are
 * a large part of a workgroup's average share (mid-length prompts with dense-like
 * heads, few heads), never pieces so short that their fixed cost shows, and never
 * more pieces than slots.  At long contexts and in launches of short rows nothing
 * exceeds L and the call equals shplb_sparse_attn_prefill.
 * Each piece is dealt to a workgroup like a row and leaves its unnormalised
 * result, reference exponent and denominator in one of `split_slots` slots of the
 * workspace (65 KB each); the piece of a row that finishes last combines the
 * row's pieces in piece order (the softmax of Eq. 1 over the union of their
 * keys) inside the same launch.  Results equal those of shplb_sparse_attn_prefill
 * up to fp32 rounding of the combination and are bit-identical from run to run.
 *   split_slots: 2 .. 65536 (4 * workgroups = 2048 never limit L).
 *   workspace: device, shplb_split_workspace_bytes(p, split_slots) bytes.
 *   Other arguments as for shplb_sparse_attn_prefill; sched_stats_out counts
 *   pieces as items.
 * Errors: SHPLB_E_UNSUPPORTED for split_slots out of range. */
SHPLB_API int32_t shplb_split_workspace_bytes(const shplb_problem* p, int32_t split_slots,
                                    int64_t* bytes_out /*host*/);
SHPLB_API int32_t shplb_sparse_attn_prefill_split(const shplb_problem* p, const void* q, const void* k,
                                        const void* v, const int64_t* sel_ptr, const int32_t* sel_idx,
                                        void* out, float* lse_out, void* sched_stats_out,
                                        void* workspace, int32_t split_slots, void* stream);

/* ---- offline profile ------------------------------------------------------- */

/* Recovery profile (Section 2.4, at the granularity the budgets count): under full
 * causal attention (Eq. 1), mass[s][h][i][j] = the attention weight that the valid
 * queries of block i put on the keys of block j, averaged over those queries, for
 * j <= i; every row sums to 1.  Entries with j > i are not written.  A dense pass
 * (every key block of every row), fp32 softmax statistics, bf16 MFMA products.
 *   q, k: device bf16.  mass_out: device fp32, laid out like the scores
 *   (shplb_score_layout()). */
SHPLB_API int32_t shplb_block_mass(const shplb_problem* p, const void* q, const void* k,
                         float* mass_out, void* stream);

/* Recovery ratio per head and budget from a block-mass profile:
 * curves_out[h][b] = mean over all queries of head h (all sequences) of the mass of
 * the b heaviest key blocks of the query's row, b = 0 .. n_levels-1; a row with
 * fewer than b visible blocks recovers all of its mass.  Non-decreasing in b: the
 * input shplb_shift_budgets takes.  All pointers are host memory.
 *   mass: host fp32 in the layout shplb_block_mass writes (copied from the device
 *   by the caller).  curves_out: [n_q_heads][n_levels] doubles, n_levels must be
 *   max blocks per sequence + 1.
 * Errors: SHPLB_E_NULL, SHPLB_E_SHAPE (also a wrong n_levels). */
SHPLB_API int32_t shplb_recovery_curves(const shplb_problem* p, const float* mass, int32_t n_levels,
                              double* curves_out);

/* Recovery ratio as the paper profiles it (Section 2.4: the cumulative attention
 * weight of a query's top-k tokens, k = 4096 there): under full causal attention
 * (Eq. 1), recovery_out[b][h][t] = the sum of the budgets[b] largest attention
 * weights of query token t of head h; a query that sees at most budgets[b] keys
 * recovers exactly 1.  Exact selection (the k-th largest weight of every query is
 * found by a bitwise search over dense sweeps, ties at the k-th place counted at
 * that weight), fp32 softmax statistics, bf16 MFMA products; a dense pass of some
 * 20 to 33 sweeps over the causal triangle: an offline tool.
 *   q, k: device bf16.  budgets: host [n_budgets], tokens, each >= 1;
 *   n_budgets: 1..SHPLB_MAX_TOKEN_BUDGETS.
 *   recovery_out: device fp32 [n_budgets][n_q_heads][T], T = cu_seqlens[n_seq].
 * Errors: SHPLB_E_NULL, SHPLB_E_SHAPE (alignment), SHPLB_E_BUDGET (a budget < 1),
 * SHPLB_E_UNSUPPORTED (n_budgets out of range). */
SHPLB_API int32_t shplb_token_recovery(const shplb_problem* p, const void* q, const void* k,
                             const int32_t* budgets /*host*/, int32_t n_budgets,
                             float* recovery_out, void* stream);

/* One figure per head and budget from shplb_token_recovery's output, as the paper
 * plots it (Section 2.4 does not say how a head's queries are combined; here: the
 * mean over all queries of the head, all sequences).  All pointers are host memory.
 *   recovery: host fp32 [n_budgets][n_q_heads][T] (copied from the device by the
 *   caller).  heads_out: [n_q_heads][n_budgets] doubles.
 * Errors: SHPLB_E_NULL, SHPLB_E_UNSUPPORTED (n_budgets out of range). */
SHPLB_API int32_t shplb_token_recovery_heads(const shplb_problem* p, const float* recovery,
                                   int32_t n_budgets, double* heads_out);

/* ---- host step ------------------------------------------------------------ */

/* Sparsity-aware head-to-partition assignment (Section 3.3, Eq. 2): visit units
 * by descending cost (equal costs: ascending index), give each to the part with
 * the smallest load so far (equal loads: lowest part index).
 * max_per_part = 0 is the paper's algorithm; > 0 additionally caps the number of
 * units per part (equal-sized GQA shares).  All pointers are host memory.
 *   costs [n] (>= 0), part_of_out [n], loads_out [n_parts] or NULL.
 * Errors: SHPLB_E_NULL; SHPLB_E_SHAPE (n < 0, n_parts < 1); SHPLB_E_BUDGET
 * (negative cost, or max_per_part * n_parts < n). */
SHPLB_API int32_t shplb_balance_heads(const int64_t* costs, int32_t n, int32_t n_parts,
                            int32_t max_per_part, int32_t* part_of_out, int64_t* loads_out);

/* Max-min sparsity budget shifting (Section 3.2): share `total` budget units
 * among the heads so that the lowest attention-weight recovery ratio is as high
 * as the iteration gets it.  Start from equal budgets (an indivisible total gives
 * its remainder to the first heads); then repeatedly move `step` units from the
 * head with the highest recovery ratio that can still give (budget - step >=
 * lower; equal ratios: lowest index) to the head with the lowest ratio (equal:
 * lowest index).  A move that would lower the minimum ratio is not made and ends
 * the iteration; a move that leaves the giver as the (possibly tied) minimum is
 * made and ends it; so does running out of givers or the receiver reaching the
 * end of its curve.  The paper fixes neither the step nor these tests.
 * All pointers are host memory.
 *   recovery [n_heads][n_levels] row-major: recovery[h][b] = ratio of head h under
 *     a budget of b units, b = 0 .. n_levels-1, non-decreasing in b.
 *   budgets_out [n_heads] (units); n_moves_out: number of moves made, or NULL.
 * The unit is the caller's (the device steps take budgets in key blocks).
 * Errors: SHPLB_E_NULL; SHPLB_E_SHAPE (n_heads < 1, n_levels < 1, step < 1,
 * lower < 0, a decreasing or non-finite curve); SHPLB_E_BUDGET (the equal start
 * lies below `lower` or beyond the curves). */
SHPLB_API int32_t shplb_shift_budgets(const double* recovery, int32_t n_heads, int32_t n_levels,
                            int64_t total, int32_t lower, int32_t step,
                            int32_t* budgets_out, int64_t* n_moves_out);

/* ---- diagnostic ------------------------------------------------------------ */

/* Rate of the bf16 matrix pipe as this chip sustains it: launches n_workgroups
 * workgroups of eight waves that issue 8 * iters v_mfma_f32_32x32x16_bf16 each on
 * register operands and nothing else.  random_operands != 0: operands with random
 * signs and mantissas and magnitudes around one (what attention multiplies);
 * 0: one small constant.  The caller times the launch (FLOP = n_workgroups * 8 *
 * 8 * iters * 32768) and may read the loop's span on workgroup 0 from scratch:
 * uint64 [0] = shader clock cycles, [1] = the same span in 100 MHz ticks.
 *   scratch: device, 16 + n_workgroups * 2048 bytes, 8-byte aligned.
 * Errors: SHPLB_E_NULL, SHPLB_E_SHAPE (iters < 1, n_workgroups < 1). */
SHPLB_API int32_t shplb_probe_mfma_rate(int32_t random_operands, int32_t iters, int32_t n_workgroups,
                              void* scratch, void* stream);

SHPLB_API const char* shplb_strerror(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* SHPLB_H */
