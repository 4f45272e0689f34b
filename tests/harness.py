"""Test-side plumbing: device buffers via torch, calls through the C-ABI binding."""
from __future__ import annotations

import numpy as np
import torch

import paper_2603_10353_amd as S
from paper_2603_10353_amd.binding import WG_STATS_DTYPE


def problem_of(wl, softmax_scale: float = 0.0) -> S.Problem:
    return S.Problem(wl.cu_seqlens, wl.n_q_heads, wl.n_kv_heads, wl.block, wl.head_dim,
                     softmax_scale=softmax_scale, kv_head_of=wl.kv_head_of)


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).to("cuda:0").view(torch.bfloat16)


def bf16_tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


class DevicePass:
    """Device-resident state of one pass of the path over a workload."""

    def __init__(self, wl, softmax_scale: float = 0.0, want_stats: bool = True, want_lse: bool = True):
        self.wl = wl
        self.p = problem_of(wl, softmax_scale)
        dev = "cuda:0"
        self.q, self.k, self.v = to_dev_bf16(wl.q), to_dev_bf16(wl.k), to_dev_bf16(wl.v)
        self.rows = S.shplb_num_rows(self.p)
        self.ws = torch.empty(S.shplb_workspace_bytes(self.p), dtype=torch.uint8, device=dev)
        self.score_off = S.shplb_score_layout(self.p)
        self.scores = torch.full((int(self.score_off[-1]),), float("nan"), dtype=torch.float32, device=dev)
        self.sel_ptr_host = S.shplb_sel_row_ptr(self.p, wl.budgets)
        self.sel_ptr = torch.from_numpy(self.sel_ptr_host).to(dev)
        self.sel_idx = torch.full((int(self.sel_ptr_host[-1]),), -1, dtype=torch.int32, device=dev)
        self.out = torch.zeros_like(self.q)
        total = self.q.shape[0]
        self.lse = torch.zeros((wl.n_q_heads, total), dtype=torch.float32, device=dev) if want_lse else None
        self.n_wg = S.shplb_sched_num_workgroups(self.p)
        self.stats = (torch.zeros(self.n_wg * WG_STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
                      if want_stats else None)

    def scores_step(self):
        S.shplb_block_scores(self.p, self.q, self.k, self.scores, self.ws, torch.cuda.current_stream())

    def select_step(self, scores=None):
        S.shplb_select_topk_per_head(self.p, self.scores if scores is None else scores, self.wl.budgets,
                                     self.sel_ptr, self.sel_idx, torch.cuda.current_stream())

    def attn_step(self, sel_ptr=None, sel_idx=None):
        S.shplb_sparse_attn_prefill(self.p, self.q, self.k, self.v,
                                    self.sel_ptr if sel_ptr is None else sel_ptr,
                                    self.sel_idx if sel_idx is None else sel_idx,
                                    self.out, self.lse, self.stats, self.ws, torch.cuda.current_stream())

    def attn_split_step(self, split_slots):
        """The attention step with long rows cut into pieces (own, larger workspace)."""
        if getattr(self, "split_slots", None) != split_slots:
            self.split_slots = split_slots
            self.ws_split = torch.empty(S.shplb_split_workspace_bytes(self.p, split_slots), dtype=torch.uint8,
                                        device="cuda:0")
        S.shplb_sparse_attn_prefill_split(self.p, self.q, self.k, self.v, self.sel_ptr, self.sel_idx, self.out,
                                          self.lse, self.stats, self.ws_split, split_slots,
                                          torch.cuda.current_stream())

    def mass_step(self):
        """Offline recovery profile into its own buffer (same layout as the scores)."""
        if not hasattr(self, "mass"):
            self.mass = torch.full_like(self.scores, float("nan"))
        S.shplb_block_mass(self.p, self.q, self.k, self.mass, torch.cuda.current_stream())

    def token_recovery_step(self, budgets):
        """Offline token-granular recovery ratio, [len(budgets), heads, tokens] on the device."""
        shape = (len(budgets), self.wl.n_q_heads, self.q.shape[0])
        if getattr(self, "token_recovery", None) is None or tuple(self.token_recovery.shape) != shape:
            self.token_recovery = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
        S.shplb_token_recovery(self.p, self.q, self.k, budgets, self.token_recovery, torch.cuda.current_stream())

    def mass_flat_host(self):
        return self.mass.cpu().numpy()

    def mass_host(self):
        flat = self.mass_flat_host()
        nbs = self.wl.n_blocks
        return [flat[self.score_off[s]:self.score_off[s + 1]].reshape(self.wl.n_q_heads, nbs[s], nbs[s])
                for s in range(self.wl.n_seq)]

    def run_all(self):
        self.scores_step()
        self.select_step()
        self.attn_step()
        torch.cuda.synchronize()
        return self

    # ---- host copies
    def scores_host(self):
        flat = self.scores.cpu().numpy()
        nbs = self.wl.n_blocks
        return [flat[self.score_off[s]:self.score_off[s + 1]].reshape(self.wl.n_q_heads, nbs[s], nbs[s])
                for s in range(self.wl.n_seq)]

    def sel_idx_host(self):
        return self.sel_idx.cpu().numpy()

    def out_host(self):
        return bf16_tensor_to_f64(self.out)

    def lse_host(self):
        return self.lse.cpu().numpy().astype(np.float64)

    def stats_host(self):
        return np.frombuffer(self.stats.cpu().numpy().tobytes(), dtype=WG_STATS_DTYPE)
