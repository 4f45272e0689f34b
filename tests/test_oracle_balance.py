"""Pins for the oracle's greedy head-to-partition assignment (paper Section 3.3, Eq. 2)."""
import itertools
import os

import numpy as np
import pytest

from oracle import shplb_oracle as orc


def _read_golden(repo_root):
    vals = {}
    with open(os.path.join(repo_root, "tests", "golden", "balance_worked_case.txt")) as f:
        for line in f:
            if line.startswith("#") or ":" not in line:
                continue
            key, rest = line.split(":", 1)
            vals[key.strip()] = [int(x) for x in rest.split()]
    return vals


def test_worked_case(repo_root):
    g = _read_golden(repo_root)
    part, loads = orc.balance_heads(g["costs"], g["n_parts"][0])
    assert part.tolist() == g["part_of"]
    assert loads.tolist() == g["loads"]
    num, den = g["imbalance_num_den"]
    assert orc.imbalance(loads) == pytest.approx(num / den, rel=1e-15)


def _optimum_max_load(costs, m):
    best = None
    for assign in itertools.product(range(m), repeat=len(costs)):
        loads = [0] * m
        for c, p in zip(costs, assign):
            loads[p] += c
        if best is None or max(loads) < best:
            best = max(loads)
    return best


@pytest.mark.parametrize("seed", range(6))
def test_greedy_vs_exhaustive_optimum(seed, repo_root):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(2, 4))
    n = int(rng.integers(m, 10))
    costs = rng.integers(1, 40, size=n).tolist()
    part, loads = orc.balance_heads(costs, m)
    # Eq. 2 constraints: every head on exactly one device, loads are budget sums
    assert sorted(np.unique(part).tolist()) == sorted(set(part.tolist())) and part.min() >= 0 and part.max() < m
    for p in range(m):
        assert loads[p] == sum(c for c, q in zip(costs, part) if q == p)
    assert loads.sum() == sum(costs)
    opt = _optimum_max_load(costs, m)
    assert opt <= loads.max() <= (4.0 / 3.0 - 1.0 / (3 * m)) * opt + 1e-9
    if seed == 0:
        g = _read_golden(repo_root)
        assert _optimum_max_load(g["costs"], 3) == g["optimum_max_load"][0]


def test_equal_costs_balance_perfectly_and_tie_breaks():
    part, loads = orc.balance_heads([7] * 12, 4)
    assert orc.imbalance(loads) == 1.0
    # equal costs keep ascending index; equal loads go to the lowest part
    assert part.tolist() == [0, 1, 2, 3] * 3


def test_greedy_beats_sequential_split_on_heterogeneous_budgets():
    # the paper's motivating observation (Section 3.2): naive sequential head
    # assignment is badly imbalanced under differentiated budgets
    rng = np.random.default_rng(123)
    worse = 0
    for _ in range(50):
        f = np.exp(rng.uniform(np.log(0.01), np.log(0.5), size=32))
        costs = np.maximum(2, np.round(f * 1024)).astype(np.int64)
        naive = costs.reshape(4, 8).sum(axis=1)
        _, loads = orc.balance_heads(costs.tolist(), 4)
        assert loads.max() <= naive.max()
        worse += orc.imbalance(naive) > 1.2
        assert orc.imbalance(loads) < 1.2
    assert worse > 25


def test_max_per_part_extension():
    rng = np.random.default_rng(7)
    costs = rng.integers(1, 1000, size=16).tolist()
    part, loads = orc.balance_heads(costs, 8, max_per_part=2)
    assert np.bincount(part, minlength=8).tolist() == [2] * 8
    assert loads.sum() == sum(costs)
    # unconstrained call on the same costs is the paper's algorithm: may differ
    part0, _ = orc.balance_heads(costs, 8)
    assert np.bincount(part0, minlength=8).sum() == 16
    with pytest.raises(ValueError):
        orc.balance_heads(costs, 4, max_per_part=3)


def test_imbalance_definition():
    assert orc.imbalance([10, 10, 10, 10]) == 1.0
    assert orc.imbalance([30, 10, 10, 10]) == 2.0
    assert orc.imbalance([1, 0]) == 2.0


def test_greedy_beats_consecutive_assignment_on_the_benchmark_layer():
    # The ablation's cost side (Section 5, Ablation Study; Eq. 2): on the 32-head layer of the 128K
    # benchmark configuration the greedy's imbalance is within 2% of perfect at 2, 4 and 8 parts,
    # while consecutive heads leave 28% (4 parts) and 100% (8 parts) on the table.
    from workloads import layer_budgets
    for seqlen in (32768, 131072):
        lb = layer_budgets(2, [seqlen])
        nb = lb["n_blocks"][0]
        k = np.clip(lb["budgets"][0].astype(np.int64), 2, nb)
        cost = k * nb - k * (k - 1) // 2
        for parts, naive_at_least in ((2, 1.0), (4, 1.25), (8, 2.0)):
            per = len(cost) // parts
            naive = orc.imbalance([int(cost[d * per:(d + 1) * per].sum()) for d in range(parts)])
            _, loads = orc.balance_heads(cost.tolist(), parts)
            assert orc.imbalance(loads) <= 1.02 and orc.imbalance(loads) <= naive
            assert naive >= naive_at_least
