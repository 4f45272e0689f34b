"""Pins for the oracle's block-sparse attention (CPU only)."""
import math

import numpy as np
import pytest
import torch

from oracle import shplb_oracle as orc
from workloads import f32_from_bf16_bits, make_custom


def _t(bits):
    return torch.from_numpy(f32_from_bf16_bits(bits).astype(np.float64))


def _sdpa_causal(wl, s):
    """Textbook routine: torch's scaled_dot_product_attention, fp64, causal, one sequence."""
    t0, t1 = int(wl.cu_seqlens[s]), int(wl.cu_seqlens[s + 1])
    g = wl.n_q_heads // wl.n_kv_heads
    q = _t(wl.q[t0:t1]).permute(1, 0, 2)                        # [Hq, S, D]
    k = _t(wl.k[t0:t1]).permute(1, 0, 2).repeat_interleave(g, dim=0)
    v = _t(wl.v[t0:t1]).permute(1, 0, 2).repeat_interleave(g, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    logits = (q @ k.transpose(1, 2)) / math.sqrt(q.shape[-1])
    mask = torch.ones(t1 - t0, t1 - t0, dtype=torch.bool).tril()
    lse = torch.logsumexp(logits.masked_fill(~mask, float("-inf")), dim=-1)
    return o.permute(1, 0, 2).numpy(), lse.numpy()


def _full_pipeline(wl):
    sc = orc.block_scores(wl.q, wl.k, wl.cu_seqlens, wl.block)
    ptr, idx = orc.select_blocks(sc, wl.budgets)
    o, lse = orc.sparse_attention(wl.q, wl.k, wl.v, wl.cu_seqlens, wl.block, ptr, idx)
    return ptr, idx, o, lse


def test_full_budget_equals_dense_causal_attention_varlen_gqa_ragged():
    # budgets >= nb for every head: the sparse path must reproduce Eq. 1 exactly,
    # per sequence (no leakage across cu_seqlens), with GQA and ragged tails.
    wl = make_custom([70, 33, 16, 5], 4, 2, 16, [99, 99, 99, 99], seed=11)
    _, _, o, lse = _full_pipeline(wl)
    assert not np.isnan(o).any() and not np.isnan(lse).any()
    for s in range(wl.n_seq):
        t0, t1 = int(wl.cu_seqlens[s]), int(wl.cu_seqlens[s + 1])
        ref_o, ref_lse = _sdpa_causal(wl, s)
        np.testing.assert_allclose(o[t0:t1], ref_o, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse[:, t0:t1], ref_lse, rtol=1e-12, atol=1e-12)


def test_budget_two_is_attention_over_sink_and_own_block():
    wl = make_custom([96], 2, 1, 16, [2, 2], seed=3)
    ptr, idx, o, _ = _full_pipeline(wl)
    q = _t(wl.q); k = _t(wl.k); v = _t(wl.v)
    for h in range(2):
        for i in range(6):
            r = h * 6 + i
            assert idx[ptr[r]:ptr[r + 1]].tolist() == ([0] if i == 0 else [0, i])
            qi = q[i * 16:(i + 1) * 16, h]
            toks = list(range(0, 16)) + ([] if i == 0 else list(range(i * 16, (i + 1) * 16)))
            kk, vv = k[toks, 0], v[toks, 0]
            mask = torch.tensor([[u <= i * 16 + r_ for u in toks] for r_ in range(16)])
            ref = torch.nn.functional.scaled_dot_product_attention(
                qi[None], kk[None], vv[None], attn_mask=mask[None])[0]
            np.testing.assert_allclose(o[i * 16:(i + 1) * 16, h], ref.numpy(), rtol=1e-11, atol=1e-12)


def test_constant_v_gives_that_constant_weights_sum_to_one():
    wl = make_custom([80, 40], 4, 2, 8, [2, 3, 4, 6], seed=4)
    const = np.linspace(-1, 1, 128).astype(np.float32)
    from workloads import bf16_bits_from_f32
    cbits = bf16_bits_from_f32(const)
    wl.v[:] = cbits[None, None, :]
    _, _, o, _ = _full_pipeline(wl)
    expect = f32_from_bf16_bits(cbits).astype(np.float64)
    assert np.abs(o - expect[None, None, :]).max() < 1e-13


def test_lse_is_log_of_softmax_denominator():
    # exp(logit - lse) over the selected, causal-visible keys must sum to one.
    wl = make_custom([64], 2, 2, 8, [3, 5], seed=8)
    ptr, idx, _, lse = _full_pipeline(wl)
    q = f32_from_bf16_bits(wl.q).astype(np.float64); k = f32_from_bf16_bits(wl.k).astype(np.float64)
    for h in range(2):
        for i in range(8):
            sel = idx[ptr[h * 8 + i]:ptr[h * 8 + i + 1]]
            for t in range(i * 8, (i + 1) * 8):
                toks = [u for j in sel for u in range(j * 8, (j + 1) * 8) if u <= t]
                logit = (k[toks, h] @ q[t, h]) / math.sqrt(128)
                assert np.exp(logit - lse[h, t]).sum() == pytest.approx(1.0, abs=1e-12)


def test_selection_order_does_not_matter():
    wl = make_custom([128], 1, 1, 16, [5], seed=9)
    ptr, idx, _, _ = _full_pipeline(wl)
    sel = idx[ptr[7]:ptr[8]]
    assert len(sel) == 5
    a, la = orc.sparse_attention_row(wl.q, wl.k, wl.v, wl.cu_seqlens, 16, 0, 0, 7, sel)
    b, lb = orc.sparse_attention_row(wl.q, wl.k, wl.v, wl.cu_seqlens, 16, 0, 0, 7, sel[::-1])
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(la, lb, rtol=1e-14)


def test_dropping_a_block_changes_the_result():
    # guards against an oracle that silently ignores the selection
    wl = make_custom([128], 1, 1, 16, [8], seed=10)
    a, _ = orc.sparse_attention_row(wl.q, wl.k, wl.v, wl.cu_seqlens, 16, 0, 0, 7, [0, 1, 2, 3, 4, 5, 6, 7])
    b, _ = orc.sparse_attention_row(wl.q, wl.k, wl.v, wl.cu_seqlens, 16, 0, 0, 7, [0, 3, 7])
    assert np.abs(a - b).max() > 1e-3
