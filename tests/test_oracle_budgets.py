"""Pins for the oracle's max-min budget shifting (Section 3.2)."""
import itertools
import os

import numpy as np
import pytest

from oracle import shplb_oracle as orc

HERE = os.path.dirname(__file__)


def _golden():
    rec, want, moves = [], None, None
    for line in open(os.path.join(HERE, "golden", "budget_shift_worked_case.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0].startswith("recovery"):
            rec.append([float(x) for x in f[1:]])
        elif f[0] == "budgets":
            want = [int(x) for x in f[1:]]
        elif f[0] == "moves":
            moves = int(f[1])
    return np.array(rec), want, moves


def test_hand_worked_instance():
    rec, want, moves = _golden()
    b, n = orc.shift_budgets(rec, total=12, lower=1, step=1)
    assert b.tolist() == want and n == moves


def test_identical_curves_keep_equal_budgets():
    curve = 1.0 - np.exp(-np.arange(40) / 7.0)
    b, n = orc.shift_budgets(np.tile(curve, (6, 1)), total=6 * 11, lower=2)
    assert b.tolist() == [11] * 6 and n == 0          # the one candidate move would lower the minimum


def test_indivisible_total_goes_to_the_first_heads():
    flat = np.ones((4, 10))
    b, _ = orc.shift_budgets(flat, total=4 * 3 + 2, lower=0)
    assert b.sum() == 14 and sorted(b.tolist(), reverse=True) == b.tolist()


def _random_curves(rng, n_heads, n_levels, plateaus):
    inc = rng.random((n_heads, n_levels)) ** rng.integers(1, 4, size=(n_heads, 1))
    if plateaus:
        inc *= rng.random((n_heads, n_levels)) < 0.6
    rec = np.cumsum(inc, axis=1)
    rec = np.concatenate([np.zeros((n_heads, 1)), rec[:, :-1]], axis=1)
    return rec / np.maximum(rec[:, -1:], 1e-9) * rng.uniform(0.5, 1.0, size=(n_heads, 1))


@pytest.mark.parametrize("plateaus", [False, True])
def test_two_heads_reach_the_exhaustive_max_min_optimum(plateaus):
    # With two heads min(R0(x), R1(total - x)) rises, then falls along x: shifting from the
    # higher to the lower head until the giver becomes the minimum must land on its maximum.
    rng = np.random.default_rng(5 + plateaus)
    for _ in range(200):
        n_levels = int(rng.integers(6, 30))
        rec = _random_curves(rng, 2, n_levels, plateaus)
        lower = int(rng.integers(0, 3))
        total = int(rng.integers(2 * lower, 2 * (n_levels - 1) + 1))
        if total // 2 < lower or (total + 1) // 2 > n_levels - 1:
            continue
        b, _ = orc.shift_budgets(rec, total, lower)
        best = max(min(rec[0][x], rec[1][total - x]) for x in range(lower, total - lower + 1)
                   if x <= n_levels - 1 and total - x <= n_levels - 1)
        got = min(rec[0][b[0]], rec[1][b[1]])
        assert b.sum() == total and b.min() >= lower
        assert got == best


def test_invariants_on_random_curves():
    rng = np.random.default_rng(11)
    for trial in range(100):
        n_heads = int(rng.integers(2, 12))
        n_levels = int(rng.integers(8, 60))
        rec = _random_curves(rng, n_heads, n_levels, plateaus=trial % 2 == 1)
        lower = int(rng.integers(0, 4))
        step = int(rng.integers(1, 3))
        per = int(rng.integers(lower, n_levels - 1))
        total = per * n_heads + int(rng.integers(0, n_heads))
        if (total + n_heads - 1) // n_heads > n_levels - 1:
            continue
        start = np.array([total // n_heads + (h < total % n_heads) for h in range(n_heads)])
        b, moves = orc.shift_budgets(rec, total, lower, step)
        assert b.sum() == total and b.min() >= lower and b.max() <= n_levels - 1
        assert np.all((b - start) % step == 0)
        r0 = min(rec[h][start[h]] for h in range(n_heads))
        r1 = [rec[h][b[h]] for h in range(n_heads)]
        assert min(r1) >= r0                                             # shifting never lowers the minimum


def test_rejects_decreasing_curves_and_bad_totals():
    rec = np.array([[0.0, 0.5, 0.4], [0.0, 0.1, 0.2]])
    with pytest.raises(ValueError):
        orc.shift_budgets(rec, 2, 0)
    ok = np.array([[0.0, 0.5, 0.6], [0.0, 0.1, 0.2]])
    with pytest.raises(ValueError):
        orc.shift_budgets(ok, 6, 0)            # 3 per head is past the curves
    with pytest.raises(ValueError):
        orc.shift_budgets(ok, 2, 2)            # below the lower bound


def test_lower_bound_stops_the_shifting():
    # Head 0 recovers everything with almost nothing, head 1 never catches up: head 0 gives
    # until it sits on the lower bound, then nobody is left to give (stopping rule ii).
    rec = np.array([[1.0] * 21, np.linspace(0.0, 0.5, 21)])
    b, n = orc.shift_budgets(rec, total=20, lower=3)
    assert b.tolist() == [3, 17] and n == 7


def test_three_heads_exhaustive_on_strictly_concave_curves():
    # Strictly concave, strictly increasing curves, no ties at the start: every move raises the
    # receiver more than it costs the giver's ranking, and the stopping state is a max-min optimum
    # over all allocations (checked exhaustively) up to one step.
    rng = np.random.default_rng(3)
    for _ in range(60):
        n_levels = 16
        rates = rng.uniform(0.08, 1.2, size=3)
        rec = 1.0 - np.exp(-np.outer(rates, np.arange(n_levels)))
        total = int(rng.integers(6, 3 * (n_levels - 1) - 3))
        if (total + 2) // 3 > n_levels - 1:
            continue
        b, _ = orc.shift_budgets(rec, total, lower=1)
        got = min(rec[h][b[h]] for h in range(3))
        best = 0.0
        for x in range(1, n_levels):
            for y in range(1, n_levels):
                z = total - x - y
                if 1 <= z <= n_levels - 1:
                    best = max(best, min(rec[0][x], rec[1][y], rec[2][z]))
        # one more unit on the weakest head is all the exhaustive optimum can be ahead by
        weakest = min(range(3), key=lambda h: rec[h][b[h]])
        one_more = rec[weakest][min(b[weakest] + 1, n_levels - 1)]
        assert got <= best <= max(got, one_more) + 1e-12
