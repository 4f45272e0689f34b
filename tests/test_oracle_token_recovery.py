"""Pins for the oracle's token-granular recovery ratio (Section 2.4: cumulative attention weight
of a query's top-k keys)."""
import itertools

import numpy as np
import torch

from oracle import shplb_oracle as orc
from workloads import bf16_bits_from_f32, make_custom


def _rand_bits(rng, shape):
    return bf16_bits_from_f32(rng.standard_normal(shape).astype(np.float32))


def test_constant_keys_closed_form():
    # all keys equal: the query at position t gives 1/(t+1) to each key it sees, so its k best hold min(k, t+1)/(t+1)
    T = 45
    rng = np.random.default_rng(0)
    q = _rand_bits(rng, (T, 2, 128))
    k = bf16_bits_from_f32(np.tile(rng.standard_normal((1, 1, 128)).astype(np.float32), (T, 1, 1)))
    budgets = [1, 4, 16, 45, 100]
    rec = orc.token_recovery(q, k, [0, T], budgets)
    t = np.arange(T)
    for b, kk in enumerate(budgets):
        want = np.minimum(kk, t + 1) / (t + 1.0)
        np.testing.assert_allclose(rec[b], np.tile(want, (2, 1)), rtol=1e-12)


def test_top_k_sums_of_a_textbook_softmax():
    wl = make_custom([150, 37], 4, 2, 32, [2, 2, 2, 2, 2, 2, 2, 2], seed=11)
    budgets = [1, 3, 20, 64]
    rec = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, budgets)
    q = torch.from_numpy(orc.decode_bf16(wl.q))
    k = torch.from_numpy(orc.decode_bf16(wl.k)).repeat_interleave(2, dim=1)
    for s in range(2):
        a, e = wl.cu_seqlens[s], wl.cu_seqlens[s + 1]
        T = e - a
        logits = torch.einsum("thd,uhd->htu", q[a:e], k[a:e]) / np.sqrt(128.0)
        logits = logits.masked_fill(torch.triu(torch.ones(T, T, dtype=torch.bool), 1), float("-inf"))
        w = torch.softmax(logits, dim=-1)                                        # [H, T, T], zeros above the diagonal
        for b, kk in enumerate(budgets):
            want = torch.topk(w, min(kk, T), dim=-1).values.sum(dim=-1).numpy()  # zeros add nothing
            np.testing.assert_allclose(rec[b][:, a:e], want, rtol=1e-10)


def test_no_subset_of_k_keys_holds_more():
    rng = np.random.default_rng(3)
    T = 9
    q, k = _rand_bits(rng, (T, 1, 128)), _rand_bits(rng, (T, 1, 128))
    budgets = [1, 2, 3, 5]
    rec = orc.token_recovery(q, k, [0, T], budgets, softmax_scale=0.3)
    qf, kf = orc.decode_bf16(q)[:, 0], orc.decode_bf16(k)[:, 0]
    for t in range(T):
        logits = kf[:t + 1] @ qf[t] * 0.3
        w = np.exp(logits) / np.exp(logits).sum()
        for b, kk in enumerate(budgets):
            best = 1.0 if kk >= t + 1 else max(sum(c) for c in itertools.combinations(w, kk))
            np.testing.assert_allclose(rec[b, 0, t], best, rtol=1e-12)


def test_one_key_is_the_largest_weight_and_more_keys_never_hold_less():
    wl = make_custom([130], 2, 1, 64, [2, 2], seed=2)
    budgets = [1, 2, 8, 32, 130, 131]
    rec = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, budgets)
    q, k = orc.decode_bf16(wl.q), orc.decode_bf16(wl.k)
    for t in (0, 1, 77, 129):
        for h in range(2):
            logits = k[:t + 1, 0] @ q[t, h] / np.sqrt(128.0)
            assert abs(rec[0, h, t] - 1.0 / np.exp(logits - logits.max()).sum()) < 1e-12
    assert (np.diff(rec, axis=0) >= -1e-15).all()
    np.testing.assert_array_equal(rec[4], 1.0)                       # budget = every key
    np.testing.assert_array_equal(rec[5], 1.0)
    assert (rec > 0).all() and (rec <= 1 + 1e-15).all()


def test_whole_blocks_of_equal_keys_agree_with_the_block_profile():
    # Keys constant inside each block of B tokens: a query's weights are equal inside a block, so for a query
    # at the end of its block its k = b*B best tokens are its b heaviest blocks (block_mass / recovery by rows).
    B, nb = 8, 6
    rng = np.random.default_rng(5)
    kb = rng.standard_normal((nb, 1, 128)).astype(np.float32)
    k = bf16_bits_from_f32(np.repeat(kb, B, axis=0))
    q = _rand_bits(rng, (nb * B, 1, 128))
    budgets = [B, 2 * B, 3 * B]
    rec = orc.token_recovery(q, k, [0, nb * B], budgets, softmax_scale=0.2)
    qf, kf = orc.decode_bf16(q)[:, 0], orc.decode_bf16(k)[:, 0]
    for i in range(nb):
        t = (i + 1) * B - 1
        logits = kf[:t + 1] @ qf[t] * 0.2
        w = np.exp(logits - logits.max())
        w /= w.sum()
        per_block = np.sort(w.reshape(i + 1, B).sum(axis=1))[::-1]
        for b in range(3):
            want = 1.0 if (b + 1) >= i + 1 else per_block[:b + 1].sum()
            np.testing.assert_allclose(rec[b, 0, t], want, rtol=1e-12)


def test_tokens_argument_and_head_means():
    wl = make_custom([70, 20], 2, 1, 32, [2, 2, 2, 2], seed=8)
    full = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, [2, 10])
    part = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, [2, 10], tokens=[0, 69, 70, 89])
    for t in range(90):
        if t in (0, 69, 70, 89):
            np.testing.assert_array_equal(part[:, :, t], full[:, :, t])
        else:
            assert np.isnan(part[:, :, t]).all()
    # the second sequence starts over: its first query sees one key
    np.testing.assert_array_equal(full[:, :, 70], 1.0)
    heads = orc.token_recovery_heads(full)
    assert heads.shape == (2, 2)
    np.testing.assert_allclose(heads[1, 0], full[0, 1].mean(), rtol=1e-15)
