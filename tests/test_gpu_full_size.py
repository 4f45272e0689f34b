"""GPU parity at the benchmark configurations' full sizes.

Scores and selections are compared on every row (the oracle's part is cheap); attention
is compared on a seeded sample of (head, query-block) rows that always contains the
costliest rows, with the oracle fed the GPU's own selection.  Properties that hold at
any size are checked on the whole output: no NaN, lse finite, scheduler bookkeeping."""
import numpy as np
import pytest
import torch

from oracle import shplb_oracle as orc
from workloads import make_workload

from checks import SCORE_ATOL, compare_output, compare_selection

pytestmark = pytest.mark.gpu


def _run_case(wl, n_sample, seed):
    from harness import DevicePass
    print("case", wl.name, "seqlens", np.diff(wl.cu_seqlens).tolist(), "heads", wl.n_q_heads, wl.n_kv_heads,
          "budgets", wl.budgets.tolist()[:8], "...", flush=True)
    run = DevicePass(wl).run_all()
    sc_o = orc.block_scores(wl.q, wl.k, wl.cu_seqlens, wl.block)
    sc_g = run.scores_host()
    for s in range(wl.n_seq):
        tri = np.tril_indices(sc_o[s].shape[1])
        for h in range(wl.n_q_heads):
            np.testing.assert_allclose(sc_g[s][h][tri], sc_o[s][h][tri], rtol=1e-5, atol=SCORE_ATOL)
    ptr_o, idx_o = orc.select_blocks(sc_o, wl.budgets)
    np.testing.assert_array_equal(ptr_o, run.sel_ptr_host)
    idx_g = run.sel_idx_host()

    def srow(r):
        s, h, i = orc.row_decode(wl.cu_seqlens, wl.block, wl.n_q_heads, r)
        return sc_o[s][h, i], i

    waived = compare_selection(ptr_o, idx_g, idx_o, srow,
                               lambda r: orc.row_decode(wl.cu_seqlens, wl.block, wl.n_q_heads, r))
    counts = np.diff(ptr_o)
    rng = np.random.default_rng(seed)
    rows = set(np.argsort(-counts, kind="stable")[:4].tolist())          # the costliest rows
    rows |= set(np.argsort(counts, kind="stable")[:2].tolist())          # and the cheapest
    first = 0
    for nb in wl.n_blocks:                                               # the costliest and the last row of every sequence
        seq_rows = np.arange(first, first + nb * wl.n_q_heads)
        rows.add(int(seq_rows[np.argmax(counts[seq_rows])]))
        rows.add(int(seq_rows[-1]))
        first += nb * wl.n_q_heads
    rows |= set(rng.choice(len(counts), size=min(n_sample, len(counts)), replace=False).tolist())
    out_o, lse_o = orc.sparse_attention(wl.q, wl.k, wl.v, wl.cu_seqlens, wl.block, ptr_o, idx_g, None, rows)
    out_g, lse_g = run.out_host(), run.lse_host()
    wa, wr, wlse = compare_output(out_g, out_o, lse_g, lse_o)
    assert np.isfinite(out_g).all() and np.isfinite(lse_g).all()
    st = run.stats_host()
    assert st["n_items"].sum() == run.rows and st["cost_blocks"].sum() == ptr_o[-1]
    busy = (st["t_last"] - st["t_first"]).astype(np.float64)
    imb = busy.max() / busy.mean() - 1.0
    print("  rows %d, waived %d, sampled %d rows: max abs %.3g max rel %.3g lse %.3g; busy-time imbalance %.3f%%"
          % (len(counts), waived, len(rows), wa, wr, wlse, 100 * imb), flush=True)
    return run, imb


def _constant_value_pass(run):
    """The attention step again with every value row of a KV head replaced by one vector w_g.
    Eq. 1 then gives O[t, h, :] = w_{g(h)} for every query, whatever was selected: a check of
    the normalisation (weights over the selected keys sum to one) and of where each result
    is written, on EVERY row of the output.  fp32 sums of p * w divided by the fp32 sum of
    the same p, then one bf16 rounding: within one bf16 step of w (2^-8 relative), plus the
    fp32 summation error, for which another half step is allowed.  The denominators do not
    depend on V, so lse must repeat the first pass bit for bit."""
    wl = run.wl
    rng = np.random.default_rng(99)
    w = torch.from_numpy(rng.uniform(0.5, 2.0, size=(wl.n_kv_heads, wl.head_dim)).astype(np.float32))
    w = (w * torch.from_numpy(rng.choice([-1.0, 1.0], size=tuple(w.shape)).astype(np.float32))).to(torch.bfloat16)
    lse_first = run.lse.clone()
    run.v[:] = w.to(run.v.device)[None]
    run.out.zero_()
    run.lse.zero_()
    run.attn_step()
    torch.cuda.synchronize()
    g = wl.n_q_heads // wl.n_kv_heads
    want = w.to(run.out.device).float().repeat_interleave(g, 0)[None]           # [1, Hq, D]
    worst = 0.0
    for t0 in range(0, run.out.shape[0], 16384):
        rel = ((run.out[t0:t0 + 16384].float() - want).abs() / want.abs()).max().item()
        worst = max(worst, rel)
    print("  constant value rows: every output row, worst relative deviation %.3g" % worst, flush=True)
    assert worst <= 1.5 * 2.0 ** -8, worst
    assert torch.equal(run.lse, lse_first)


def test_config1_32k_full():
    run, imb = _run_case(make_workload(1), 48, seed=1)
    assert imb < 0.05
    _constant_value_pass(run)


def test_config2_128k_full():
    run, imb = _run_case(make_workload(2), 24, seed=2)
    assert imb < 0.05
    _constant_value_pass(run)


def test_config3_one_partition_share_64k():
    import paper_2603_10353_amd as S
    import bench
    heads, loads = bench.pick_config3_heads(S)
    run, imb = _run_case(make_workload(3, q_heads=heads), 32, seed=3)
    # 8 heads, 4096 rows on 512 workgroups: eight items per workgroup, the coarsest case of the set
    assert imb < 0.08


def test_config4_varlen_batch_quarter_scale():
    # the 8K+24K+64K+128K batch at a quarter of its lengths (ragged by one token each), one launch
    _run_case(make_workload(4, seqlens=[2048 + 1, 6144 - 1, 16384 + 63, 32768 - 65]), 48, seed=4)


def test_config4_varlen_batch_full():
    # 8K + 24K + 64K + 128K tokens in one launch: 57 344 rows of four sequences go through the
    # five-launch ordering (two counting sorts with multi-sequence row decoding) into one
    # persistent attention launch.  Scores and selections on every row; attention on sampled
    # rows that include the costliest and the last row of every sequence; then every output row
    # through the constant-value check.
    run, imb = _run_case(make_workload(4), 48, seed=5)
    assert imb < 0.05
    _constant_value_pass(run)


def test_block64_32k_layer():
    # The 32K layer with 64-token blocks and the same budgets in tokens (twice as many blocks): 16 384 rows
    # of up to 256 blocks through the 64-token instance of the pipelined kernel (32-key tiles, four
    # workgroups per compute unit).
    from workloads import layer_budgets, make_custom
    budgets = 2 * layer_budgets(1, [32768])["budgets"][0]
    wl = make_custom([32768], 32, 8, 64, [int(x) for x in budgets], seed=5, c_range=(0.25, 6.0), name="layer32k_b64")
    run, imb = _run_case(wl, 40, seed=9)
    assert imb < 0.05
    _constant_value_pass(run)


def test_three_sequences_above_the_single_workgroup_ordering():
    # 17 024 rows (> 16 384, where the single-workgroup ordering ends) from three ragged sequences
    # of a 64/16-head layer: the five-launch ordering with multi-sequence decoding at a size where
    # the sample can be dense (1 row in 70) and the oracle still finishes in seconds.
    from workloads import make_custom
    rng = np.random.default_rng(123)
    budgets = rng.choice([2, 3, 5, 9, 17, 40, 999], size=3 * 64)
    wl = make_custom([128 * 120 + 17, 128 * 90 - 5, 128 * 54 + 1], 64, 16, 128, budgets, seed=79, name="three_seq")
    run, imb = _run_case(wl, 240, seed=6)
    assert run.rows > 16384
    _constant_value_pass(run)


def test_max_blocks_per_sequence():
    # 4096 blocks of 64 tokens: the largest block count the library accepts (wide selection kernel,
    # score tiles in rounds, 64-token attention kernel at scale); the last block is ragged.
    from workloads import make_custom
    wl = make_custom([64 * 4096 - 37], 2, 1, 64, [48, 700], seed=77, name="max_blocks")
    _run_case(wl, 12, seed=7)


def test_max_sequences_per_call():
    # 64 sequences (the most one call takes), lengths from one token to a few blocks, GQA 4:1.
    from workloads import make_custom
    rng = np.random.default_rng(64)
    seqlens = [1, 127, 128, 129] + rng.integers(1, 900, size=60).tolist()
    wl = make_custom(seqlens, 8, 2, 128, [1, 2, 3, 4, 6, 9, 2, 100], seed=78, name="max_seq")
    _run_case(wl, 64, seed=8)
