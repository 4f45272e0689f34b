"""Pins for the oracle's recovery profile (Section 2.4 at block granularity)."""
import numpy as np
import pytest
import torch

from oracle import shplb_oracle as orc
from workloads import bf16_bits_from_f32, make_custom


def test_rows_sum_to_one_and_nothing_above_the_diagonal():
    wl = make_custom([300, 64, 1, 129], 4, 2, 64, [3, 3, 3, 3], seed=5)
    for m in orc.block_mass(wl.q, wl.k, wl.cu_seqlens, wl.block):
        nb = m.shape[1]
        for i in range(nb):
            np.testing.assert_allclose(m[:, i, :i + 1].sum(axis=1), 1.0, rtol=0, atol=1e-12)
            assert np.isnan(m[:, i, i + 1:]).all()
        assert (m[~np.isnan(m)] >= 0).all()


def test_constant_keys_closed_form():
    # All keys equal: every query spreads its weight evenly over the keys it sees.  Query at
    # position t gives 1/(t+1) to each; block j < i collects B/(t+1), the diagonal block the rest.
    B, T = 16, 16 * 5 + 7
    rng = np.random.default_rng(0)
    q = bf16_bits_from_f32(rng.standard_normal((T, 2, 128)).astype(np.float32))
    k = bf16_bits_from_f32(np.tile(rng.standard_normal((1, 1, 128)).astype(np.float32), (T, 1, 1)))
    m = orc.block_mass(q, k, [0, T], B)[0]
    nb = m.shape[1]
    for i in range(nb):
        ts = np.arange(i * B, min((i + 1) * B, T))
        for j in range(i):
            np.testing.assert_allclose(m[:, i, j], np.mean(B / (ts + 1.0)), rtol=1e-12)
        np.testing.assert_allclose(m[:, i, i], np.mean((ts - i * B + 1.0) / (ts + 1.0)), rtol=1e-12)


def test_block_sums_of_a_textbook_softmax():
    wl = make_custom([200], 4, 2, 32, [2, 2, 2, 2], seed=9)
    q = torch.from_numpy(orc.decode_bf16(wl.q))
    k = torch.from_numpy(orc.decode_bf16(wl.k)).repeat_interleave(2, dim=1)
    T, B = 200, 32
    logits = torch.einsum("thd,uhd->htu", q, k) / np.sqrt(128.0)
    logits = logits.masked_fill(torch.triu(torch.ones(T, T, dtype=torch.bool), 1), float("-inf"))
    w = torch.softmax(logits, dim=-1).numpy()                                   # [H, T, T]
    m = orc.block_mass(wl.q, wl.k, wl.cu_seqlens, B)[0]
    nb = m.shape[1]
    for i in range(nb):
        for j in range(i + 1):
            want = w[:, i * B:(i + 1) * B, j * B:(j + 1) * B].sum(axis=(1, 2)) / (min((i + 1) * B, T) - i * B)
            np.testing.assert_allclose(m[:, i, j], want, rtol=1e-10, atol=1e-14)


def test_rows_argument_limits_the_work():
    wl = make_custom([256, 100], 2, 1, 64, [2, 2], seed=3)
    full = orc.block_mass(wl.q, wl.k, wl.cu_seqlens, 64)
    rows = [0, 5, 9, 11]
    part = orc.block_mass(wl.q, wl.k, wl.cu_seqlens, 64, rows=rows)
    seen = 0
    for s in range(2):
        for h in range(2):
            for i in range(full[s].shape[1]):
                r = orc.row_index(wl.cu_seqlens, 64, 2, s, h, i)
                if r in rows:
                    np.testing.assert_array_equal(part[s][h, i, :i + 1], full[s][h, i, :i + 1])
                    seen += 1
                else:
                    assert np.isnan(part[s][h, i]).all()
    assert seen == len(rows)


def test_recovery_curves_closed_forms():
    # One sequence of 4 full blocks.  Head 0: every row spreads its mass evenly over its visible
    # blocks (row i recovers min(b, i+1)/(i+1)); head 1: all mass on one block (recovers 1 from b = 1).
    nb = 4
    m = np.full((2, nb, nb), np.nan)
    for i in range(nb):
        m[0, i, :i + 1] = 1.0 / (i + 1)
        m[1, i, :i + 1] = 0.0
        m[1, i, i // 2] = 1.0
    c = orc.recovery_curves([m], [0, 4 * 8], 8)
    assert c.shape == (2, nb + 1)
    for b in range(nb + 1):
        assert c[0, b] == pytest.approx(np.mean([min(b, i + 1) / (i + 1) for i in range(nb)]))
        assert c[1, b] == pytest.approx(0.0 if b == 0 else 1.0)


def test_recovery_curves_weight_rows_by_their_queries_and_are_concave():
    wl = make_custom([64 * 6 + 10, 40], 4, 2, 64, [2, 2, 2, 2], seed=21)
    mass = orc.block_mass(wl.q, wl.k, wl.cu_seqlens, 64)
    c = orc.recovery_curves(mass, wl.cu_seqlens, 64)
    assert np.all(c[:, 0] == 0) and np.allclose(c[:, -1], 1.0)
    d = np.diff(c, axis=1)
    assert (d >= -1e-15).all() and (np.diff(d, axis=1) <= 1e-12).all()          # heaviest first: increments shrink
    # budget 1 recovers, per row, its heaviest block: check the query weighting by hand
    cu = [int(x) for x in wl.cu_seqlens]
    tot = np.zeros(4)
    nq = 0
    for s, nb in enumerate(orc.blocks_per_sequence(cu, 64)):
        for i in range(nb):
            n_valid = min(64, cu[s + 1] - cu[s] - i * 64)
            nq += n_valid
            tot += n_valid * np.nanmax(mass[s][:, i, :], axis=1)
    np.testing.assert_allclose(c[:, 1], tot / nq, rtol=1e-12)


def test_selection_recovery_of_everything_is_one_and_of_the_best_blocks_is_the_curve():
    wl = make_custom([64 * 5 + 3], 2, 1, 64, [3, 3], seed=8)
    mass = orc.block_mass(wl.q, wl.k, wl.cu_seqlens, 64)
    nb = mass[0].shape[1]
    ptr = orc.sel_row_ptr(wl.cu_seqlens, 64, 2, [nb, nb])
    idx = np.concatenate([np.arange(i + 1) for _h in range(2) for i in range(nb)]).astype(np.int32)
    np.testing.assert_allclose(orc.selection_recovery(mass, wl.cu_seqlens, 64, ptr, idx), 1.0, atol=1e-12)
    ptr2 = orc.sel_row_ptr(wl.cu_seqlens, 64, 2, [2, 2])
    best = []
    for h in range(2):
        for i in range(nb):
            best.append(np.sort(np.argsort(-mass[0][h, i, :i + 1], kind="stable")[:min(2, i + 1)]))
    idx2 = np.concatenate(best).astype(np.int32)
    c = orc.recovery_curves(mass, wl.cu_seqlens, 64)
    np.testing.assert_allclose(orc.selection_recovery(mass, wl.cu_seqlens, 64, ptr2, idx2), c[:, 2], rtol=1e-12)
