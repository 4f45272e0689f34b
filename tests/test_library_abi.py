"""CPU-side checks of the boundary: the library loads, exports what the header
declares, validates arguments, and the host-side entry points agree with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2603_10353_amd as S
from paper_2603_10353_amd.binding import EXPORTS
from oracle import shplb_oracle as orc


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(S.lib_path()):
        from paper_2603_10353_amd.build import build
        build(verbose=False)


def test_exports_match_header(repo_root):
    hdr = open(os.path.join(repo_root, "include", "shplb.h")).read()
    declared = sorted(set(re.findall(r"SHPLB_API\s+[\w\s\*]+?\b(shplb_\w+)\s*\(", hdr)))
    assert declared == sorted(EXPORTS)
    lib = S.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layout_matches_header():
    from paper_2603_10353_amd.binding import _CProblem, WgStats
    assert C.sizeof(_CProblem) == 80 and _CProblem.softmax_scale.offset == 64 and _CProblem.kv_head_of.offset == 72
    assert C.sizeof(WgStats) == 32


def test_shape_helpers_against_oracle():
    cu = [0, 300, 301, 1000]
    p = S.Problem(cu, 8, 2, 64)
    nbs = orc.blocks_per_sequence(cu, 64)
    assert S.shplb_num_rows(p) == 8 * sum(nbs)
    off = S.shplb_score_layout(p)
    assert off.tolist() == [0] + np.cumsum([8 * nb * nb for nb in nbs]).tolist()
    rng = np.random.default_rng(0)
    budgets = rng.integers(0, 20, size=3 * 8)
    np.testing.assert_array_equal(S.shplb_sel_row_ptr(p, budgets), orc.sel_row_ptr(cu, 64, 8, budgets))
    assert S.shplb_workspace_bytes(p) > 0


def test_argument_validation():
    ok = dict(cu_seqlens=[0, 128], n_q_heads=4, n_kv_heads=2, block=128)

    def status(**kw):
        args = dict(ok); args.update(kw)
        try:
            S.shplb_num_rows(S.Problem(**args))
            return 0
        except S.ShplbError as e:
            return e.status
    assert status() == 0
    assert status(head_dim=64) == -5
    assert status(block=32) == -5
    assert status(n_q_heads=3) == -2
    assert status(cu_seqlens=[1, 128]) == -2
    assert status(cu_seqlens=[0, 128, 128]) == -2
    assert status(cu_seqlens=list(range(0, 66 * 128, 128))) == -5       # 65 sequences
    assert status(cu_seqlens=[0, 128 * 4097]) == -5                      # too many blocks
    assert status(q_stride_h=100) == -2
    assert status(q_stride_h=132) == -2                                  # not 16-byte aligned
    assert status(softmax_scale=-1.0) == -2
    p = S.Problem(**ok)
    with pytest.raises(S.ShplbError) as e:
        S.shplb_sel_row_ptr(p, [1, 2, -1, 3])
    assert e.value.status == -3
    # null device pointers are rejected before any device work
    with pytest.raises(S.ShplbError) as e:
        S.shplb_block_scores(p, None, None, None, None)
    assert e.value.status == -1
    with pytest.raises(S.ShplbError) as e:
        S.shplb_sparse_attn_prefill(p, None, None, None, None, None, None)
    assert e.value.status == -1
    with pytest.raises(S.ShplbError) as e:
        S.shplb_select_topk_per_head(p, None, [2, 2, 2, 2], None, None)
    assert e.value.status == -1
    # the split variant: the slot count is checked on the host, before anything else
    assert S.shplb_split_workspace_bytes(p, 64) > S.shplb_workspace_bytes(p) + 64 * 65536
    for bad in (0, 1, -5, 65537):
        with pytest.raises(S.ShplbError) as e:
            S.shplb_split_workspace_bytes(p, bad)
        assert e.value.status == -5
        with pytest.raises(S.ShplbError) as e:
            S.shplb_sparse_attn_prefill_split(p, None, None, None, None, None, None, split_slots=bad)
        assert e.value.status == -5
    p64 = S.Problem(**dict(ok, block=64))
    assert S.shplb_split_workspace_bytes(p64, 64) > S.shplb_workspace_bytes(p64) + 64 * 65536
    with pytest.raises(S.ShplbError) as e:
        S.shplb_sparse_attn_prefill_split(p, None, None, None, None, None, None, split_slots=64)
    assert e.value.status == -1
    assert "null" in S.shplb_strerror(-1) and S.shplb_strerror(0) == "ok"
    # an explicit query-head -> KV-head map lifts the divisibility rule and is range-checked
    assert S.shplb_num_rows(S.Problem([0, 1000], 5, 2, 128, kv_head_of=[0, 0, 1, 0, 1])) == 5 * 8
    for bad in ([0, 0, 2, 0, 1], [0, -1, 1, 0, 1]):
        with pytest.raises(S.ShplbError) as e:
            S.shplb_num_rows(S.Problem([0, 1000], 5, 2, 128, kv_head_of=bad))
        assert e.value.status == -2
    with pytest.raises(S.ShplbError) as e:
        S.shplb_num_rows(S.Problem([0, 1000], 300, 2, 128, kv_head_of=[0] * 300))
    assert e.value.status == -5
    with pytest.raises(S.ShplbError) as e:
        S.shplb_num_rows(S.Problem([0, 1000], 5, 2, 128))           # no map: 5 heads do not divide into 2 groups
    assert e.value.status == -2


@pytest.mark.parametrize("seed", range(8))
def test_balance_heads_bit_exact_vs_oracle(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 65))
    parts = int(rng.integers(1, 9))
    costs = rng.integers(0, 50 if seed % 2 else 100000, size=n)      # small range => many ties
    part, loads = S.shplb_balance_heads(costs, parts)
    po, lo = orc.balance_heads(costs.tolist(), parts)
    np.testing.assert_array_equal(part, po)
    np.testing.assert_array_equal(loads, lo)
    cap = -(-n // parts)
    part, loads = S.shplb_balance_heads(costs, parts, cap)
    po, lo = orc.balance_heads(costs.tolist(), parts, cap)
    np.testing.assert_array_equal(part, po)
    np.testing.assert_array_equal(loads, lo)
    assert np.bincount(part, minlength=parts).max() <= cap


def test_balance_heads_errors_and_golden(repo_root):
    part, loads = S.shplb_balance_heads([5, 5, 4, 4, 3, 3, 3], 3)
    assert part.tolist() == [0, 1, 2, 2, 0, 1, 0] and loads.tolist() == [11, 8, 8]
    for bad, code in [(dict(costs=[1, 2], n_parts=0), -2), (dict(costs=[1, -2], n_parts=2), -3),
                      (dict(costs=[1, 2, 3], n_parts=2, max_per_part=1), -3)]:
        with pytest.raises(S.ShplbError) as e:
            S.shplb_balance_heads(**bad)
        assert e.value.status == code
    part, loads = S.shplb_balance_heads([], 3)
    assert part.size == 0 and loads.tolist() == [0, 0, 0]


def test_config3_share_selection():
    # 16 KV groups of the 64-head layer -> 8 parts of 2 groups (equal-sized shares)
    import bench
    heads, loads = bench.pick_config3_heads(S)
    assert len(heads) == 8 and heads[0] % 4 == 0 and heads[4] % 4 == 0
    assert orc.imbalance(loads) < 1.35


def _monotone_curves(rng, n_heads, n_levels):
    inc = rng.random((n_heads, n_levels)) ** rng.integers(1, 4, size=(n_heads, 1))
    inc *= rng.random((n_heads, n_levels)) < 0.7                      # plateaus: exact ties between heads and steps
    rec = np.cumsum(inc, axis=1)
    return np.round(rec / np.maximum(rec[:, -1:], 1e-9) * rng.uniform(0.5, 1.0, size=(n_heads, 1)), 3)


@pytest.mark.parametrize("seed", range(6))
def test_shift_budgets_bit_exact_vs_oracle(seed):
    rng = np.random.default_rng(300 + seed)
    for _ in range(60):
        n_heads = int(rng.integers(1, 40))
        n_levels = int(rng.integers(4, 300))
        rec = _monotone_curves(rng, n_heads, n_levels)
        lower = int(rng.integers(0, 4))
        step = int(rng.integers(1, 4))
        total = int(rng.integers(lower, n_levels - 1)) * n_heads + int(rng.integers(0, n_heads))
        try:
            bo, mo = orc.shift_budgets(rec, total, lower, step)
        except ValueError:
            with pytest.raises(S.ShplbError):
                S.shplb_shift_budgets(rec, total, lower, step)
            continue
        bg, mg = S.shplb_shift_budgets(rec, total, lower, step)
        np.testing.assert_array_equal(bg, bo)
        assert mg == mo


def test_shift_budgets_golden_and_errors(repo_root):
    rec = [[0.00, 0.50, 0.80, 0.90, 0.95, 0.97, 0.98, 0.99, 1.00],
           [0.00, 0.10, 0.20, 0.30, 0.40, 0.50, 0.60, 0.70, 0.80],
           [0.00, 0.30, 0.55, 0.70, 0.80, 0.86, 0.90, 0.93, 0.95]]
    b, n = S.shplb_shift_budgets(rec, 12, 1)
    assert b.tolist() == [2, 6, 4] and n == 2
    for bad, status in [(dict(recovery=[[0.0, 0.5, 0.4]], total=1, lower=0), -2),       # decreasing curve
                        (dict(recovery=[[0.0, float("nan")]], total=1, lower=0), -2),
                        (dict(recovery=rec, total=12, lower=1, step=0), -2),
                        (dict(recovery=rec, total=30, lower=1), -3),                    # 10 per head: past the curves
                        (dict(recovery=rec, total=3, lower=2), -3)]:                    # below the lower bound
        with pytest.raises(S.ShplbError) as e:
            S.shplb_shift_budgets(**bad)
        assert e.value.status == status


def test_recovery_curves_vs_oracle_on_host():
    # Host entry point fed the oracle's own block masses (as fp32, in the library's layout).
    from workloads import make_custom
    wl = make_custom([64 * 5 + 9, 30, 64 * 2], 4, 2, 64, [2, 2, 2, 2], seed=44)
    mass = orc.block_mass(wl.q, wl.k, wl.cu_seqlens, 64)
    p = S.Problem(wl.cu_seqlens, 4, 2, 64)
    flat = np.concatenate([np.nan_to_num(m, nan=0.0).astype(np.float32).reshape(-1) for m in mass])
    got = S.shplb_recovery_curves(p, flat)
    want = orc.recovery_curves([m.astype(np.float32).astype(np.float64) for m in mass], wl.cu_seqlens, 64)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)
    with pytest.raises(ValueError):
        S.shplb_recovery_curves(p, flat[:-1])


def test_token_recovery_host_side():
    # the per-head mean is host work; the device entry point checks its arguments before any launch
    from workloads import make_custom
    wl = make_custom([70, 33], 4, 2, 64, [2] * 8, seed=45)
    rec = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, [1, 5, 40]).astype(np.float32)
    p = S.Problem(wl.cu_seqlens, 4, 2, 64)
    got = S.shplb_token_recovery_heads(p, rec)
    np.testing.assert_allclose(got, orc.token_recovery_heads(rec.astype(np.float64)), rtol=1e-12)
    with pytest.raises(ValueError):
        S.shplb_token_recovery_heads(p, rec[:, :, :-1])
    with pytest.raises(S.ShplbError) as e:
        S.shplb_token_recovery(p, None, None, [4], None)
    assert e.value.status == -1
    fake = 4096                                            # never dereferenced: rejected on the host
    for budgets, status in (([0], -3), ([4, -1], -3), ([], -5), (list(range(1, 10)), -5)):
        with pytest.raises(S.ShplbError) as e:
            S.shplb_token_recovery(p, fake, fake, budgets, fake)
        assert e.value.status == status, budgets


def test_header_is_plain_c_and_a_c_program_links(tmp_path):
    # the boundary is a C ABI: the header must compile as C99, and a C caller must link and run the host entry points
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                    os.path.join(inc, "shplb.h")], check=True)
    src = tmp_path / "caller.c"
    src.write_text(r'''
#include <stdio.h>
#include "shplb.h"
int main(void) {
  /* the worked instance of list scheduling on three machines */
  const int64_t costs[7] = {5, 5, 4, 4, 3, 3, 3};
  int32_t part_of[7];
  int64_t loads[3];
  if (shplb_balance_heads(costs, 7, 3, 0, part_of, loads) != SHPLB_OK) return 1;
  if (loads[0] != 11 || loads[1] != 8 || loads[2] != 8) return 2;
  int32_t cu[2] = {0, 1000};
  shplb_problem p = {1, cu, 8, 2, 128, 128, 8 * 128, 128, 2 * 128, 128, 0.0f, 0};
  int64_t rows = 0;
  if (shplb_num_rows(&p, &rows) != SHPLB_OK || rows != 8 * 8) return 3;
  printf("%s\n", shplb_strerror(SHPLB_E_BUDGET));
  return 0;
}
''')
    exe = tmp_path / "caller"
    lib = S.lib_path()
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), lib,
                    "-Wl,-rpath," + os.path.dirname(lib)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True)
    assert out.stdout.strip() != ""
