"""ctypes marshalling for libshplb.so.  No arithmetic of the method lives here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = [
    "shplb_num_rows", "shplb_max_blocks", "shplb_workspace_bytes", "shplb_score_layout", "shplb_sel_row_ptr",
    "shplb_sched_num_workgroups", "shplb_block_scores", "shplb_select_topk_per_head",
    "shplb_sparse_attn_prefill", "shplb_sparse_attn_prefill_static", "shplb_split_workspace_bytes", "shplb_sparse_attn_prefill_split",
    "shplb_balance_heads", "shplb_shift_budgets", "shplb_block_mass",
    "shplb_recovery_curves", "shplb_token_recovery", "shplb_token_recovery_heads", "shplb_probe_mfma_rate",
    "shplb_strerror",
]


class ShplbError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: status %d (%s)" % (where, status, shplb_strerror(status)))


class _CProblem(C.Structure):
    _fields_ = [
        ("n_seq", C.c_int32),
        ("cu_seqlens", C.POINTER(C.c_int32)),
        ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32),
        ("block", C.c_int32),
        ("q_stride_t", C.c_int64),
        ("q_stride_h", C.c_int64),
        ("kv_stride_t", C.c_int64),
        ("kv_stride_h", C.c_int64),
        ("softmax_scale", C.c_float),
        ("kv_head_of", C.POINTER(C.c_int32)),
    ]


class WgStats(C.Structure):
    _fields_ = [
        ("xcc_id", C.c_uint32),
        ("cu_id", C.c_uint32),
        ("n_items", C.c_uint32),
        ("cost_blocks", C.c_uint32),
        ("t_first", C.c_uint64),
        ("t_last", C.c_uint64),
    ]


WG_STATS_DTYPE = np.dtype([("xcc_id", "<u4"), ("cu_id", "<u4"), ("n_items", "<u4"),
                           ("cost_blocks", "<u4"), ("t_first", "<u8"), ("t_last", "<u8")])


def lib_path() -> str:
    """Path of the shared library: SHPLB_LIBRARY if set, else the in-tree build."""
    return os.environ.get("SHPLB_LIBRARY") or os.path.join(_PKG, "libshplb.so")


def load_library():
    """Load libshplb.so from the package directory.  Raises if it has not been built
    (python -m paper_2603_10353_amd.build); there is no fallback implementation."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("libshplb.so is not built: run `python -m paper_2603_10353_amd.build` "
                          "(hipcc, gfx950). No CPU fallback exists.")
    lib = C.CDLL(path)
    i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
    pp = C.POINTER(_CProblem)
    lib.shplb_num_rows.argtypes = [pp, C.POINTER(i64)]
    lib.shplb_max_blocks.argtypes = [pp, C.POINTER(i32)]
    lib.shplb_workspace_bytes.argtypes = [pp, C.POINTER(i64)]
    lib.shplb_score_layout.argtypes = [pp, C.POINTER(i64)]
    lib.shplb_sel_row_ptr.argtypes = [pp, C.POINTER(i32), C.POINTER(i64)]
    lib.shplb_sched_num_workgroups.argtypes = [pp, C.POINTER(i32)]
    lib.shplb_block_scores.argtypes = [pp, vp, vp, vp, vp, vp]
    lib.shplb_select_topk_per_head.argtypes = [pp, vp, C.POINTER(i32), vp, vp, vp]
    lib.shplb_sparse_attn_prefill.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.shplb_sparse_attn_prefill_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.shplb_split_workspace_bytes.argtypes = [pp, i32, C.POINTER(i64)]
    lib.shplb_sparse_attn_prefill_split.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
    lib.shplb_balance_heads.argtypes = [C.POINTER(i64), i32, i32, i32, C.POINTER(i32), C.POINTER(i64)]
    lib.shplb_probe_mfma_rate.argtypes = [i32, i32, i32, vp, vp]
    lib.shplb_block_mass.argtypes = [pp, vp, vp, vp, vp]
    lib.shplb_recovery_curves.argtypes = [pp, C.POINTER(C.c_float), i32, C.POINTER(C.c_double)]
    lib.shplb_token_recovery.argtypes = [pp, vp, vp, C.POINTER(C.c_int32), i32, vp, vp]
    lib.shplb_token_recovery_heads.argtypes = [pp, C.POINTER(C.c_float), i32, C.POINTER(C.c_double)]
    lib.shplb_shift_budgets.argtypes = [C.POINTER(C.c_double), i32, i32, i64, i32, i32, C.POINTER(i32),
                                        C.POINTER(i64)]
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = i32
    lib.shplb_strerror.argtypes = [i32]
    lib.shplb_strerror.restype = C.c_char_p
    _LIB = lib
    return lib


class Problem:
    """Host-side mirror of the C struct shplb_problem (keeps cu_seqlens and kv_head_of alive)."""

    def __init__(self, cu_seqlens: Sequence[int], n_q_heads: int, n_kv_heads: int, block: int,
                 head_dim: int = 128, q_stride_t: Optional[int] = None, q_stride_h: Optional[int] = None,
                 kv_stride_t: Optional[int] = None, kv_stride_h: Optional[int] = None,
                 softmax_scale: float = 0.0, kv_head_of: Optional[Sequence[int]] = None):
        self.cu = np.ascontiguousarray(np.asarray(cu_seqlens, dtype=np.int32))
        self.kv_head_of = None if kv_head_of is None else np.ascontiguousarray(np.asarray(kv_head_of, dtype=np.int32))
        if self.kv_head_of is not None and self.kv_head_of.size != n_q_heads:
            raise ValueError("kv_head_of must hold n_q_heads entries")
        q_stride_h = head_dim if q_stride_h is None else q_stride_h
        kv_stride_h = head_dim if kv_stride_h is None else kv_stride_h
        q_stride_t = n_q_heads * q_stride_h if q_stride_t is None else q_stride_t
        kv_stride_t = n_kv_heads * kv_stride_h if kv_stride_t is None else kv_stride_t
        self.c = _CProblem(len(self.cu) - 1, self.cu.ctypes.data_as(C.POINTER(C.c_int32)),
                           n_q_heads, n_kv_heads, head_dim, block, q_stride_t, q_stride_h,
                           kv_stride_t, kv_stride_h, softmax_scale,
                           None if self.kv_head_of is None else self.kv_head_of.ctypes.data_as(C.POINTER(C.c_int32)))

    @property
    def n_seq(self) -> int:
        return self.c.n_seq

    @property
    def n_q_heads(self) -> int:
        return self.c.n_q_heads

    def ref(self):
        return C.byref(self.c)


def _dev(x) -> Optional[int]:
    """Device pointer of a tensor-like (anything with data_ptr()), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _check(status: int, where: str):
    if status != 0:
        raise ShplbError(status, where)


def shplb_strerror(status: int) -> str:
    return load_library().shplb_strerror(int(status)).decode()


def shplb_num_rows(p: Problem) -> int:
    out = C.c_int64()
    _check(load_library().shplb_num_rows(p.ref(), C.byref(out)), "shplb_num_rows")
    return out.value


def shplb_max_blocks(p: Problem) -> int:
    out = C.c_int32()
    _check(load_library().shplb_max_blocks(p.ref(), C.byref(out)), "shplb_max_blocks")
    return out.value


def shplb_workspace_bytes(p: Problem) -> int:
    out = C.c_int64()
    _check(load_library().shplb_workspace_bytes(p.ref(), C.byref(out)), "shplb_workspace_bytes")
    return out.value


def shplb_score_layout(p: Problem) -> np.ndarray:
    out = np.zeros(p.n_seq + 1, np.int64)
    _check(load_library().shplb_score_layout(p.ref(), out.ctypes.data_as(C.POINTER(C.c_int64))),
           "shplb_score_layout")
    return out


def shplb_sel_row_ptr(p: Problem, budgets) -> np.ndarray:
    b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32))
    if b.size != p.n_seq * p.n_q_heads:
        raise ValueError("budgets must hold n_seq * n_q_heads entries")
    out = np.zeros(shplb_num_rows(p) + 1, np.int64)
    _check(load_library().shplb_sel_row_ptr(p.ref(), b.ctypes.data_as(C.POINTER(C.c_int32)),
                                            out.ctypes.data_as(C.POINTER(C.c_int64))), "shplb_sel_row_ptr")
    return out


def shplb_sched_num_workgroups(p: Problem) -> int:
    out = C.c_int32()
    _check(load_library().shplb_sched_num_workgroups(p.ref(), C.byref(out)), "shplb_sched_num_workgroups")
    return out.value


def shplb_block_scores(p: Problem, q, k, scores_out, workspace, stream=None) -> None:
    _check(load_library().shplb_block_scores(p.ref(), _dev(q), _dev(k), _dev(scores_out), _dev(workspace),
                                             _stream(stream)), "shplb_block_scores")


def shplb_select_topk_per_head(p: Problem, scores, budgets, sel_ptr, sel_idx_out, stream=None) -> None:
    b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32))
    if b.size != p.n_seq * p.n_q_heads:
        raise ValueError("budgets must hold n_seq * n_q_heads entries")
    _check(load_library().shplb_select_topk_per_head(p.ref(), _dev(scores), b.ctypes.data_as(C.POINTER(C.c_int32)),
                                                     _dev(sel_ptr), _dev(sel_idx_out), _stream(stream)),
           "shplb_select_topk_per_head")


def shplb_sparse_attn_prefill(p: Problem, q, k, v, sel_ptr, sel_idx, out, lse_out=None,
                              sched_stats_out=None, workspace=None, stream=None) -> None:
    _check(load_library().shplb_sparse_attn_prefill(p.ref(), _dev(q), _dev(k), _dev(v), _dev(sel_ptr),
                                                    _dev(sel_idx), _dev(out), _dev(lse_out),
                                                    _dev(sched_stats_out), _dev(workspace), _stream(stream)),
           "shplb_sparse_attn_prefill")


def shplb_sparse_attn_prefill_static(p: Problem, q, k, v, sel_ptr, sel_idx, out, lse_out=None,
                                     sched_stats_out=None, stream=None) -> None:
    _check(load_library().shplb_sparse_attn_prefill_static(p.ref(), _dev(q), _dev(k), _dev(v), _dev(sel_ptr),
                                                           _dev(sel_idx), _dev(out), _dev(lse_out),
                                                           _dev(sched_stats_out), _stream(stream)),
           "shplb_sparse_attn_prefill_static")


def shplb_split_workspace_bytes(p: Problem, split_slots: int) -> int:
    out = C.c_int64(0)
    _check(load_library().shplb_split_workspace_bytes(p.ref(), int(split_slots), C.byref(out)),
           "shplb_split_workspace_bytes")
    return int(out.value)


def shplb_sparse_attn_prefill_split(p: Problem, q, k, v, sel_ptr, sel_idx, out, lse_out=None,
                                    sched_stats_out=None, workspace=None, split_slots: int = 0,
                                    stream=None) -> None:
    _check(load_library().shplb_sparse_attn_prefill_split(p.ref(), _dev(q), _dev(k), _dev(v), _dev(sel_ptr),
                                                          _dev(sel_idx), _dev(out), _dev(lse_out),
                                                          _dev(sched_stats_out), _dev(workspace),
                                                          int(split_slots), _stream(stream)),
           "shplb_sparse_attn_prefill_split")


def shplb_balance_heads(costs, n_parts: int, max_per_part: int = 0):
    """Returns (part_of int32 [n], loads int64 [n_parts])."""
    c = np.ascontiguousarray(np.asarray(costs, dtype=np.int64))
    part = np.zeros(c.size, np.int32)
    loads = np.zeros(max(int(n_parts), 0), np.int64)
    _check(load_library().shplb_balance_heads(c.ctypes.data_as(C.POINTER(C.c_int64)), c.size, int(n_parts),
                                              int(max_per_part), part.ctypes.data_as(C.POINTER(C.c_int32)),
                                              loads.ctypes.data_as(C.POINTER(C.c_int64)) if n_parts > 0 else None),
           "shplb_balance_heads")
    return part, loads


def shplb_shift_budgets(recovery, total: int, lower: int, step: int = 1):
    """recovery: [n_heads, n_levels] float64.  Returns (budgets int32 [n_heads], number of moves)."""
    r = np.ascontiguousarray(np.asarray(recovery, dtype=np.float64))
    if r.ndim != 2:
        raise ValueError("recovery must be [n_heads, n_levels]")
    budgets = np.zeros(r.shape[0], np.int32)
    moves = C.c_int64(0)
    _check(load_library().shplb_shift_budgets(r.ctypes.data_as(C.POINTER(C.c_double)), r.shape[0], r.shape[1],
                                              int(total), int(lower), int(step),
                                              budgets.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(moves)),
           "shplb_shift_budgets")
    return budgets, int(moves.value)


def shplb_block_mass(p: Problem, q, k, mass_out, stream=None) -> None:
    _check(load_library().shplb_block_mass(p.ref(), _dev(q), _dev(k), _dev(mass_out), _stream(stream)),
           "shplb_block_mass")


def shplb_recovery_curves(p: Problem, mass_host) -> np.ndarray:
    """mass_host: float32 host array in the layout shplb_block_mass writes.  Returns float64 [n_q_heads, max_nb + 1]."""
    m = np.ascontiguousarray(np.asarray(mass_host, dtype=np.float32)).reshape(-1)
    off = shplb_score_layout(p)
    if m.size != int(off[-1]):
        raise ValueError("mass has %d floats, layout needs %d" % (m.size, int(off[-1])))
    n_levels = shplb_max_blocks(p) + 1
    curves = np.zeros((p.c.n_q_heads, n_levels), np.float64)
    _check(load_library().shplb_recovery_curves(p.ref(), m.ctypes.data_as(C.POINTER(C.c_float)), n_levels,
                                                curves.ctypes.data_as(C.POINTER(C.c_double))),
           "shplb_recovery_curves")
    return curves


def shplb_token_recovery(p: Problem, q, k, budgets, recovery_out, stream=None) -> None:
    """budgets: host int32 [n_budgets] (tokens); recovery_out: device float32 [n_budgets, n_q_heads, T]."""
    b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32)).reshape(-1)
    _check(load_library().shplb_token_recovery(p.ref(), _dev(q), _dev(k), b.ctypes.data_as(C.POINTER(C.c_int32)),
                                               int(b.size), _dev(recovery_out), _stream(stream)),
           "shplb_token_recovery")


def shplb_token_recovery_heads(p: Problem, recovery_host) -> np.ndarray:
    """recovery_host: float32 host array [n_budgets, n_q_heads, T].  Returns float64 [n_q_heads, n_budgets]."""
    r = np.ascontiguousarray(np.asarray(recovery_host, dtype=np.float32))
    if r.ndim != 3 or r.shape[1] != p.c.n_q_heads or r.shape[2] != int(p.cu[-1]):
        raise ValueError("recovery must be [n_budgets, n_q_heads, T]")
    heads = np.zeros((p.c.n_q_heads, r.shape[0]), np.float64)
    _check(load_library().shplb_token_recovery_heads(p.ref(), r.ctypes.data_as(C.POINTER(C.c_float)), int(r.shape[0]),
                                                     heads.ctypes.data_as(C.POINTER(C.c_double))),
           "shplb_token_recovery_heads")
    return heads


def shplb_probe_mfma_rate(random_operands: bool, iters: int, n_workgroups: int, scratch, stream=None) -> None:
    _check(load_library().shplb_probe_mfma_rate(int(bool(random_operands)), int(iters), int(n_workgroups),
                                                _dev(scratch), _stream(stream)), "shplb_probe_mfma_rate")
