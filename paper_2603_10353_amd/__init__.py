"""S-HPLB hot path on one MI355X: head-adaptive block-sparse causal prefill.

Thin ctypes binding over libshplb.so (hand-written HIP for gfx950).  The functions
carry the names of the C entry points declared in include/shplb.h and only marshal
arguments; every step of the path runs in the library's kernels.  There is no CPU
fallback: importing works without the library, calling does not.
"""
from .binding import (  # noqa: F401
    Problem,
    ShplbError,
    WgStats,
    lib_path,
    load_library,
    shplb_balance_heads,
    shplb_block_mass,
    shplb_block_scores,
    shplb_max_blocks,
    shplb_num_rows,
    shplb_probe_mfma_rate,
    shplb_recovery_curves,
    shplb_sched_num_workgroups,
    shplb_score_layout,
    shplb_sel_row_ptr,
    shplb_shift_budgets,
    shplb_select_topk_per_head,
    shplb_sparse_attn_prefill,
    shplb_sparse_attn_prefill_split,
    shplb_sparse_attn_prefill_static,
    shplb_split_workspace_bytes,
    shplb_strerror,
    shplb_token_recovery,
    shplb_token_recovery_heads,
    shplb_workspace_bytes,
)
