"""Pins for the oracle's pooling, scoring and selection (CPU only)."""
import itertools
import math

import numpy as np
import pytest

from oracle import shplb_oracle as orc
from workloads import bf16_bits_from_f32, make_custom, make_workload


def _bits(x):
    return bf16_bits_from_f32(np.asarray(x, np.float32))


def test_decode_bf16_exact_values():
    # 1.0, -2.0, 0.5, 3.140625 (0x4049) as bf16 patterns
    bits = np.array([0x3F80, 0xC000, 0x3F00, 0x4049], np.uint16)
    np.testing.assert_array_equal(orc.decode_bf16(bits), [1.0, -2.0, 0.5, 3.140625])


def test_scores_closed_form_constant_blocks():
    # Q block i is the constant a_i in every coordinate, K block j the constant b_j:
    # pooled dot = a_i * b_j * D, so s = a_i * b_j * D / sqrt(D) = a_i * b_j * sqrt(D).
    blk, nb, d = 4, 5, 128
    a = np.array([1, 2, -1, 3, 0.5])
    b = np.array([2, -1, 4, 0.25, 1])
    q = np.repeat(a, blk)[:, None, None] * np.ones((1, 1, d))
    k = np.repeat(b, blk)[:, None, None] * np.ones((1, 1, d))
    sc = orc.block_scores(_bits(q), _bits(k), [0, blk * nb], blk)[0]
    for i in range(nb):
        for j in range(nb):
            if j <= i:
                assert sc[0, i, j] == pytest.approx(a[i] * b[j] * math.sqrt(d), rel=1e-14)
            else:
                assert np.isnan(sc[0, i, j])


def test_scores_one_hot_and_explicit_scale():
    # Q block i = e_i, K block j = e_j (one-hot coordinates): score = [i == j] * scale
    blk, nb, d = 2, 6, 128
    q = np.zeros((blk * nb, 1, d)); k = np.zeros((blk * nb, 1, d))
    for i in range(nb):
        q[i * blk:(i + 1) * blk, 0, i] = 1.0
        k[i * blk:(i + 1) * blk, 0, i] = 1.0
    sc = orc.block_scores(_bits(q), _bits(k), [0, blk * nb], blk, scale=0.25)[0][0]
    tri = np.tril_indices(nb)
    np.testing.assert_array_equal(sc[tri], 0.25 * np.eye(nb)[tri])


def test_pool_ragged_tail_is_mean_over_valid_tokens_and_sequences_do_not_mix():
    # two sequences of 5 and 3 tokens, block 4: blocks {4,1} and {3} tokens.
    d = 128
    x = np.zeros((8, 1, d))
    x[:, 0, 0] = [1, 2, 3, 6, 10, 100, 200, 300]
    pooled = orc.pool_blocks(_bits(x), [0, 5, 8], 4)
    assert pooled[0].shape == (1, 2, d) and pooled[1].shape == (1, 1, d)
    assert pooled[0][0, 0, 0] == 3.0          # (1+2+3+6)/4
    assert pooled[0][0, 1, 0] == 10.0         # one valid token, not diluted by padding
    assert pooled[1][0, 0, 0] == 200.0        # (100+200+300)/3, nothing from sequence 0


def test_scores_gqa_head_uses_its_group():
    # KV head g has every key equal to (g+1) in coordinate 0; Q is e_0 everywhere.
    blk, nb, d, hq, hkv = 2, 3, 128, 4, 2
    q = np.zeros((blk * nb, hq, d)); q[:, :, 0] = 1.0
    k = np.zeros((blk * nb, hkv, d))
    for g in range(hkv):
        k[:, g, 0] = g + 1
    sc = orc.block_scores(_bits(q), _bits(k), [0, blk * nb], blk, scale=1.0)[0]
    for h in range(hq):
        assert sc[h, 2, 1] == (h // 2) + 1


# ------------------------------------------------------------------ selection
def _brute_force_row(scores_row, i, n):
    """Best n-subset of {0..i} containing {0,i}: maximal candidate score sum; among
    equal sums the lexicographically smallest index tuple (= lower index wins)."""
    forced = {0, i}
    cands = [j for j in range(1, i)]
    want = n - len(forced)
    best = None
    for combo in itertools.combinations(cands, want):
        key = (-sum(float(scores_row[j]) for j in combo), combo)
        if best is None or key < best[0]:
            best = (key, combo)
    return np.array(sorted(forced | set(best[1])), np.int32)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_select_matches_brute_force_on_tiny_rows(seed):
    rng = np.random.default_rng(seed)
    nb = 9
    # few distinct values => plenty of exact ties; integers keep subset sums exact
    sc = rng.integers(-2, 3, size=(2, nb, nb)).astype(np.float64)
    for k in range(0, nb + 2):
        ptr, idx = orc.select_blocks([sc], [k, max(k - 1, 0)])
        r = 0
        for h, kh in enumerate([k, max(k - 1, 0)]):
            for i in range(nb):
                n = orc.n_selected(kh, nb, i)
                got = idx[ptr[r]:ptr[r + 1]]
                np.testing.assert_array_equal(got, _brute_force_row(sc[h, i], i, n))
                r += 1


def test_select_constructed_ties_take_lower_index():
    nb = 8
    row = np.array([9, 1, 5, 5, 5, 1, 5, 9], np.float64)   # candidates 1..6 for i=7
    # n=4 -> two picks among the four 5s at j=2,3,4,6 -> 2 and 3
    np.testing.assert_array_equal(orc.select_row(row, 7, 4), [0, 2, 3, 7])
    # n=6 -> all of 2,3,4,6
    np.testing.assert_array_equal(orc.select_row(row, 7, 6), [0, 2, 3, 4, 6, 7])
    # n=7 -> plus the lower-index 1.0 (j=1, not j=5)
    np.testing.assert_array_equal(orc.select_row(row, 7, 7), [0, 1, 2, 3, 4, 6, 7])


def test_select_signed_zero_is_a_tie():
    row = np.array([0, -0.0, 0.0, -1.0, 7], np.float32)
    np.testing.assert_array_equal(orc.select_row(row, 4, 3), [0, 1, 4])
    row = np.array([0, 0.0, -0.0, -1.0, 7], np.float32)
    np.testing.assert_array_equal(orc.select_row(row, 4, 3), [0, 1, 4])


def test_select_forced_blocks_and_budget_clamp():
    nb = 6
    sc = np.zeros((1, nb, nb)); sc[0, :, 3] = 100.0; sc[0, :, 0] = -100.0
    for k in (0, 1, 2):   # budgets below two still keep sink + diagonal
        ptr, idx = orc.select_blocks([sc], [k])
        rows = [idx[ptr[r]:ptr[r + 1]].tolist() for r in range(nb)]
        assert rows == [[0], [0, 1], [0, 2], [0, 3], [0, 4], [0, 5]]
    ptr, idx = orc.select_blocks([sc], [3])
    assert idx[ptr[5]:ptr[6]].tolist() == [0, 3, 5]
    assert idx[ptr[4]:ptr[5]].tolist() == [0, 3, 4]
    ptr, idx = orc.select_blocks([sc], [1000])   # above nb: everything causal-visible
    assert idx[ptr[5]:ptr[6]].tolist() == [0, 1, 2, 3, 4, 5]


@pytest.mark.parametrize("k,nb", [(2, 4), (5, 32), (32, 32), (1, 7), (100, 9), (26, 256)])
def test_row_ptr_total_closed_form(k, nb):
    # sum_{i<nb} min(k', i+1) = k' nb - k'(k'-1)/2 with k' = clamp(k, 2, nb)
    ptr = orc.sel_row_ptr([0, nb * 16], 16, 1, [k])
    kk = min(max(k, 2), nb)
    assert ptr[-1] == kk * nb - kk * (kk - 1) // 2
    assert (np.diff(ptr) == [min(kk, i + 1) for i in range(nb)]).all()


def test_row_ptr_matches_select_and_row_index_roundtrip():
    wl = make_custom([100, 37, 64], 4, 2, 16, [2, 3, 5, 9], seed=5)
    sc = orc.block_scores(wl.q, wl.k, wl.cu_seqlens, wl.block)
    ptr, idx = orc.select_blocks(sc, wl.budgets)
    np.testing.assert_array_equal(ptr, orc.sel_row_ptr(wl.cu_seqlens, wl.block, 4, wl.budgets))
    nbs = orc.blocks_per_sequence(wl.cu_seqlens, wl.block)
    assert nbs == [7, 3, 4]
    r = 0
    for s, nb in enumerate(nbs):
        for h in range(4):
            for i in range(nb):
                assert orc.row_index(wl.cu_seqlens, wl.block, 4, s, h, i) == r
                assert orc.row_decode(wl.cu_seqlens, wl.block, 4, r) == (s, h, i)
                r += 1


def test_select_invariants_on_config0():
    wl = make_workload(0)
    sc = orc.block_scores(wl.q, wl.k, wl.cu_seqlens, wl.block)
    ptr, idx = orc.select_blocks(sc, wl.budgets)
    nb = 32
    r = 0
    planted_seen = planted_hit = 0
    for h in range(wl.n_q_heads):
        k = int(wl.budgets[h])
        for i in range(nb):
            sel = idx[ptr[r]:ptr[r + 1]]
            assert len(sel) == min(max(k, 2), i + 1)
            assert sel[0] == 0 and sel[-1] == i
            assert (np.diff(sel) > 0).all()
            chosen = set(sel.tolist()) - {0, i}
            rest = [j for j in range(1, i) if j not in chosen]
            if chosen and rest:
                lo = min(sc[0][h, i, j] for j in chosen)
                assert max(sc[0][h, i, j] for j in rest) <= lo
                for j in rest:          # an equal score may lose only to a lower index
                    if sc[0][h, i, j] == lo:
                        assert j > max(jj for jj in chosen if sc[0][h, i, jj] == lo)
            # generator sanity: planted heavy blocks win when visible and affordable
            if k >= 4 and 1.4 * wl.meta["conc"][h] > 0.5:
                for hb in wl.meta["heavy"][0, h]:
                    if 0 < hb < i:
                        planted_seen += 1
                        planted_hit += int(hb in chosen)
            r += 1
    assert planted_seen > 50 and planted_hit == planted_seen
