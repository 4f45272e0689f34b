"""GPU parity: HIP path through the C-ABI vs the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import shplb_oracle as orc
from workloads import make_custom, make_workload

from checks import SCORE_ATOL, compare_output, compare_selection

pytestmark = pytest.mark.gpu


def _gpu():
    from harness import DevicePass
    return DevicePass


def full_parity(wl, softmax_scale=0.0, rows=None):
    """scores, selection (with the near-threshold waiver), attention (oracle fed the
    GPU's own selection) and lse, all rows unless `rows` is given."""
    print("case", wl.name, "seqlens", np.diff(wl.cu_seqlens).tolist(), "heads", wl.n_q_heads, wl.n_kv_heads,
          "block", wl.block, "budgets", wl.budgets.tolist()[:16], flush=True)
    run = _gpu()(wl, softmax_scale).run_all()
    if wl.kv_head_of is not None:
        # the oracle knows equal groups only: it gets every query head's K/V head as a head of its own
        from workloads import one_kv_head_per_query_head
        wl = one_kv_head_per_query_head(wl)
    scale = None if softmax_scale == 0.0 else softmax_scale
    sc_o = orc.block_scores(wl.q, wl.k, wl.cu_seqlens, wl.block, scale)
    sc_g = run.scores_host()
    for s in range(wl.n_seq):
        tri = np.tril_indices(sc_o[s].shape[1])
        for h in range(wl.n_q_heads):
            np.testing.assert_allclose(sc_g[s][h][tri], sc_o[s][h][tri], rtol=1e-5, atol=SCORE_ATOL)
            up = np.triu_indices(sc_o[s].shape[1], 1)
            assert np.isnan(sc_g[s][h][up]).all(), "entries above the diagonal must stay unwritten"
    ptr_o, idx_o = orc.select_blocks(sc_o, wl.budgets)
    np.testing.assert_array_equal(ptr_o, run.sel_ptr_host)
    idx_g = run.sel_idx_host()

    def srow(r):
        s, h, i = orc.row_decode(wl.cu_seqlens, wl.block, wl.n_q_heads, r)
        return sc_o[s][h, i], i

    waived = compare_selection(ptr_o, idx_g, idx_o, srow,
                               lambda r: orc.row_decode(wl.cu_seqlens, wl.block, wl.n_q_heads, r))
    out_o, lse_o = orc.sparse_attention(wl.q, wl.k, wl.v, wl.cu_seqlens, wl.block, ptr_o, idx_g, scale, rows)
    wa, wr, wl_ = compare_output(run.out_host(), out_o, run.lse_host(), lse_o)
    print("  waived rows %d / %d, out max abs %.3g max rel %.3g, lse max abs %.3g" % (waived, len(ptr_o) - 1, wa, wr, wl_),
          flush=True)
    return run


def test_config0_full():
    run = full_parity(make_workload(0))
    st = run.stats_host()
    assert st["n_items"].sum() == run.rows
    assert st["cost_blocks"].sum() == run.sel_ptr_host[-1]


@pytest.mark.parametrize("block", [64, 128])
def test_gqa_ragged_varlen(block):
    # several tiles, ragged tails, a one-token sequence, a sequence shorter than a block
    wl = make_custom([5 * block + 37, 1, block - 3, 2 * block, 3 * block + 1], 8, 2, block,
                     [0, 1, 2, 3, 4, 5, 7, 100], seed=21 + block, name="ragged_b%d" % block)
    full_parity(wl)


@pytest.mark.parametrize("heads", [(28, 4), (40, 8), (12, 2), (5, 5), (3, 1)])
def test_group_sizes_of_the_evaluated_models(heads):
    # GQA groups that are no powers of two (the Qwen2.5 models of Section 5.1 have 28/4, 40/8 and 64/8 heads),
    # MHA with an odd head count, and one KV head for all
    hq, hkv = heads
    budgets = [2 + (5 * h) % 9 for h in range(hq)]
    full_parity(make_custom([700, 130], hq, hkv, 128, budgets, seed=300 + hq, name="heads_%d_%d" % heads))


def test_config1_shape_scaled_down():
    # Llama-3-8B-shaped GQA layer (32/8 heads, block 128) at 4K tokens + a ragged tail
    full_parity(make_workload(1, seqlens=[4096 + 77]))


def test_dense_budget_equals_dense_attention():
    wl = make_custom([1024 + 50], 4, 1, 128, [999] * 4, seed=31, name="dense")
    run = full_parity(wl)
    # independent check against a textbook routine on the GPU result itself
    from workloads import f32_from_bf16_bits
    q = torch.from_numpy(f32_from_bf16_bits(wl.q).astype(np.float64)).permute(1, 0, 2)
    k = torch.from_numpy(f32_from_bf16_bits(wl.k).astype(np.float64)).permute(1, 0, 2).repeat_interleave(4, 0)
    v = torch.from_numpy(f32_from_bf16_bits(wl.v).astype(np.float64)).permute(1, 0, 2).repeat_interleave(4, 0)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True).permute(1, 0, 2).numpy()
    compare_output(run.out_host(), ref)


def test_long_and_short_rows_mixed():
    # Rows of up to 41 selected blocks beside rows of 2 or 3: dense, wide and narrow heads, a
    # ragged tail, a second shorter sequence, GQA.  Work items of very different length go
    # through the queues together; every selected block is visited exactly once.
    wl = make_custom([128 * 40 + 37, 128 * 11], 4, 2, 128, [999, 999, 23, 3, 999, 18, 2, 7], seed=61, name="mixed")
    run = full_parity(wl)
    st = run.stats_host()
    assert st["cost_blocks"].sum() == run.sel_ptr_host[-1]
    assert st["n_items"].sum() == run.rows


def _split_against_whole_rows(wl, split_slots, min_pieces_of_longest):
    """shplb_sparse_attn_prefill_split against the oracle (like the plain entry point) and against
    the plain entry point's own output; twice, for run-to-run identity."""
    run = _gpu()(wl).run_all()
    o_plain, l_plain = run.out.clone(), run.lse.clone()
    run.out.zero_(); run.lse.zero_()
    run.attn_split_step(split_slots)
    torch.cuda.synchronize()
    sc_o = orc.block_scores(wl.q, wl.k, wl.cu_seqlens, wl.block, None)
    ptr_o, _ = orc.select_blocks(sc_o, wl.budgets)
    out_o, lse_o = orc.sparse_attention(wl.q, wl.k, wl.v, wl.cu_seqlens, wl.block, ptr_o, run.sel_idx_host(), None, None)
    wa, wr, wl_ = compare_output(run.out_host(), out_o, run.lse_host(), lse_o)
    st = run.stats_host()
    print("  %s split_slots %d: items %d for %d rows, out max abs %.3g max rel %.3g lse %.3g" % (
        wl.name, split_slots, st["n_items"].sum(), run.rows, wa, wr, wl_), flush=True)
    assert st["cost_blocks"].sum() == run.sel_ptr_host[-1]      # every selected block visited exactly once
    # more items than rows: pieces; the longest row alone accounts for its share of the extra ones
    assert st["n_items"].sum() >= run.rows + min_pieces_of_longest - 1
    if min_pieces_of_longest == 1:
        assert st["n_items"].sum() == run.rows
        assert torch.equal(run.out.view(torch.int16), o_plain.view(torch.int16)) and torch.equal(run.lse, l_plain)
    # against the unsplit result: the same sums in another order
    d = (run.out.float() - o_plain.float()).abs().max().item()
    assert d <= 2.0 ** -6, d
    assert (run.lse - l_plain).abs().max().item() <= 2e-3       # denominators are sums of bf16-rounded probabilities
    o1, l1 = run.out.clone(), run.lse.clone()
    run.out.zero_(); run.lse.zero_()
    run.attn_split_step(split_slots)
    torch.cuda.synchronize()
    assert torch.equal(run.out.view(torch.int16), o1.view(torch.int16))   # neither slot numbers nor who merges matter
    assert torch.equal(run.lse, l1)
    return run


@pytest.mark.parametrize("split_slots", [128, 1024])
def test_long_rows_split_along_keys_and_merged(split_slots):
    # The mixed case above through shplb_sparse_attn_prefill_split: 2741 selected blocks.  With 1024
    # slots every row of more than 16 blocks is cut (the 41-block rows into 3 pieces), with 128 slots
    # only rows of more than 43 would be: none, and the call must equal the plain one bit for bit.
    # The piece of a row that finishes last merges.
    wl = make_custom([128 * 40 + 37, 128 * 11], 4, 2, 128, [999, 999, 23, 3, 999, 18, 2, 7], seed=61, name="split")
    _split_against_whole_rows(wl, split_slots, 3 if split_slots == 1024 else 1)


def test_split_rows_block_64_many_pieces():
    # 64-token blocks (the non-pipelined kernel): rows of up to 141 blocks are cut into up to five
    # pieces of at least 32 blocks; GQA, ragged tail, a second sequence of one block
    wl = make_custom([64 * 140 + 21, 50], 4, 2, 64, [999, 70, 2, 9, 999, 3, 5, 999], seed=62, name="split64")
    _split_against_whole_rows(wl, 2048, 5)


def test_split_leaves_short_rows_whole():
    # configuration 0 (8 heads, 2K tokens, block 64): no row reaches the shortest piece length, so the
    # split entry point must do exactly what the plain one does
    wl = make_workload(0)
    run = _gpu()(wl).run_all()
    o_plain, l_plain = run.out.clone(), run.lse.clone()
    run.out.zero_(); run.lse.zero_()
    run.attn_split_step(1024)
    torch.cuda.synchronize()
    assert run.stats_host()["n_items"].sum() == run.rows
    assert torch.equal(run.out.view(torch.int16), o_plain.view(torch.int16)) and torch.equal(run.lse, l_plain)


@pytest.mark.parametrize("block", [64, 128])
def test_packed_qkv_strides(block):
    # Q, K, V as column slices of one [T, Hq + 2 Hkv, 128] buffer (the output of a fused QKV
    # projection), O into a buffer with the strides of Q: only the addressing differs from the
    # contiguous case, so scores, selection, output and lse must come out bit-identical to it,
    # and the contiguous case is what the oracle checks.
    import paper_2603_10353_amd as S
    from harness import to_dev_bf16
    wl = make_custom([128 * 9 + 77, 300], 6, 2, block, [5, 999, 3, 7, 2, 4] * 2, seed=71, name="packed")
    ref = full_parity(wl)
    hq, hkv, d = wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    width = hq + 2 * hkv
    packed = torch.empty((ref.q.shape[0], width, d), dtype=torch.bfloat16, device="cuda:0")
    packed[:, :hq] = to_dev_bf16(wl.q)
    packed[:, hq:hq + hkv] = to_dev_bf16(wl.k)
    packed[:, hq + hkv:] = to_dev_bf16(wl.v)
    q, k, v = packed[:, :hq], packed[:, hq:hq + hkv], packed[:, hq + hkv:]
    out_buf = torch.zeros_like(packed)
    out = out_buf[:, :hq]
    p = S.Problem(wl.cu_seqlens, hq, hkv, block, d, q_stride_t=width * d, q_stride_h=d,
                  kv_stride_t=width * d, kv_stride_h=d)
    ws = torch.empty(S.shplb_workspace_bytes(p), dtype=torch.uint8, device="cuda:0")
    scores = torch.full_like(ref.scores, float("nan"))
    sel_idx = torch.full_like(ref.sel_idx, -1)
    lse = torch.zeros_like(ref.lse)
    st = torch.cuda.current_stream()
    S.shplb_block_scores(p, q, k, scores, ws, st)
    S.shplb_select_topk_per_head(p, scores, wl.budgets, ref.sel_ptr, sel_idx, st)
    S.shplb_sparse_attn_prefill(p, q, k, v, ref.sel_ptr, sel_idx, out, lse, None, ws, st)
    torch.cuda.synchronize()
    assert torch.equal(torch.nan_to_num(scores, nan=-7.0), torch.nan_to_num(ref.scores, nan=-7.0))
    assert torch.equal(sel_idx, ref.sel_idx)
    assert torch.equal(out.contiguous().view(torch.int16), ref.out.view(torch.int16))
    assert torch.equal(lse, ref.lse)
    assert not out_buf[:, hq:].any()                    # nothing written outside the O columns


@pytest.mark.parametrize("block", [64, 128])
def test_caller_supplied_selection_sink_and_window(block):
    # The attention step on a selection that did not come from the selection kernel: every row
    # keeps block 0 and a window of its last w_h blocks (ascending, contains the diagonal), the
    # window differing per head; the first rows have a single block.  Ragged tail, two sequences.
    wl = make_custom([block * 21 + 13, block * 2 + 1], 4, 2, block, [2] * 8, seed=81, name="window")
    run = _gpu()(wl)
    windows = [1, 2, 5, 30]
    ptr, idx = [0], []
    for s, nb in enumerate(wl.n_blocks):
        for h in range(wl.n_q_heads):
            for i in range(nb):
                sel = sorted({0} | set(range(max(0, i - windows[h] + 1), i + 1)))
                idx += sel
                ptr.append(len(idx))
    ptr, idx = np.asarray(ptr, np.int64), np.asarray(idx, np.int32)
    run.attn_step(torch.from_numpy(ptr).to("cuda:0"), torch.from_numpy(idx).to("cuda:0"))
    torch.cuda.synchronize()
    out_o, lse_o = orc.sparse_attention(wl.q, wl.k, wl.v, wl.cu_seqlens, wl.block, ptr, idx, None, None)
    wa, wr, wl_ = compare_output(run.out_host(), out_o, run.lse_host(), lse_o)
    st = run.stats_host()
    assert st["cost_blocks"].sum() == len(idx) and st["n_items"].sum() == run.rows
    print("  window selection: out max abs %.3g max rel %.3g" % (wa, wr), flush=True)


def test_whole_path_in_a_hip_graph():
    # The three entry points captured into one HIP graph (kernel launches only, no memset nodes: the
    # ordering kernels clear their own counters) and replayed several times with eager work
    # and synchronisations in between; every replay must reproduce the eager result bit for bit.
    wl = make_workload(1, seqlens=[128 * 37 + 5])
    run = _gpu()(wl).run_all()                       # eager pass: reference, and warms up every lazy init
    ref = (run.scores.clone(), run.sel_idx.clone(), run.out.clone(), run.lse.clone())
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run.scores_step(); run.select_step(); run.attn_step()      # once on the side stream before capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run.scores_step()
            run.select_step()
            run.attn_step()
    torch.cuda.synchronize()
    for replay in range(4):
        run.scores.fill_(float("nan")); run.sel_idx.fill_(-1); run.out.zero_(); run.lse.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        nan = lambda t: torch.nan_to_num(t, nan=-7.0)
        assert torch.equal(nan(run.scores), nan(ref[0])), replay
        assert torch.equal(run.sel_idx, ref[1]), replay
        assert torch.equal(run.out.view(torch.int16), ref[2].view(torch.int16)), replay
        assert torch.equal(run.lse, ref[3]), replay


@pytest.mark.parametrize("block", [64, 128])
def test_irregular_share_of_heads(block):
    # A device's share under the head-to-device assignment: query heads 0, 3, 4, 5, 7, 9 of a 12/4-head
    # layer (groups of 3) read KV heads 0, 1, 1, 1, 2, 3 -- groups of 1, 3, 1 and 1 heads, which only an
    # explicit map can express.  Two ragged sequences.
    from workloads import take_heads
    layer = make_custom([block * 9 + 31, block * 3 + 2], 12, 4, block, [2, 999, 5, 3, 7, 4, 999, 2, 6, 5, 3, 8] * 2,
                        seed=97, name="layer12")
    share = take_heads(layer, [0, 3, 4, 5, 7, 9])
    assert share.kv_head_of.tolist() == [0, 1, 1, 1, 2, 3] and share.n_kv_heads == 4
    run = full_parity(share)
    # the shared run must agree bit for bit with the same heads run with private K/V copies
    from workloads import one_kv_head_per_query_head
    ref = _gpu()(one_kv_head_per_query_head(share)).run_all()
    assert torch.equal(run.out.view(torch.int16), ref.out.view(torch.int16)) and torch.equal(run.lse, ref.lse)
    assert torch.equal(run.sel_idx, ref.sel_idx)


def test_explicit_softmax_scale():
    wl = make_custom([700], 2, 2, 64, [3, 6], seed=41, name="scale")
    full_parity(wl, softmax_scale=0.05)


def test_select_kernel_bit_exact_on_given_scores():
    # Same fp32 scores on both sides, many exact ties: lists must be identical.
    wl = make_custom([64 * 70, 64 * 9 + 5], 4, 4, 64, [2, 5, 17, 64, 3, 9, 33, 1], seed=51, name="ties")
    run = _gpu()(wl)
    rng = np.random.default_rng(5)
    nbs = wl.n_blocks
    sc = [rng.integers(-3, 4, size=(4, nb, nb)).astype(np.float32) * 0.25 for nb in nbs]
    sc[0][0, :, 3] = -0.0
    sc[0][0, :, 5] = 0.0
    flat = np.concatenate([x.reshape(-1) for x in sc])
    run.select_step(torch.from_numpy(flat).to("cuda:0"))
    torch.cuda.synchronize()
    ptr_o, idx_o = orc.select_blocks(sc, wl.budgets)
    np.testing.assert_array_equal(run.sel_ptr_host, ptr_o)
    np.testing.assert_array_equal(run.sel_idx_host(), idx_o)


def test_select_kernel_on_scores_of_one_sign_and_of_extreme_range():
    # The search runs inside the sign that holds the threshold, on keys relative to that sign's smallest:
    # rows of one sign only, rows with exactly the wanted number of non-negative scores, magnitudes from
    # denormals to 1e30, and distinct values throughout (no ties to hide behind).
    nb = 300
    budgets = [2, 3, 12, 40, 130, 299, 7, 77]
    wl = make_custom([64 * nb], 8, 8, 64, budgets, seed=52, name="signs")
    run = _gpu()(wl)
    rng = np.random.default_rng(6)
    sc = np.zeros((8, nb, nb), np.float32)
    mag = lambda shape: np.exp(rng.uniform(np.log(1e-30), np.log(1e30), size=shape)).astype(np.float32)
    sc[0] = -mag((nb, nb))                                   # all negative
    sc[1] = mag((nb, nb))                                    # all positive
    sc[2] = rng.standard_normal((nb, nb)).astype(np.float32) * 1e-40   # denormals of both signs
    sc[3] = rng.standard_normal((nb, nb)).astype(np.float32)
    for h in (4, 5, 6, 7):                                   # exactly want = k - 2 non-negative candidates per row
        want = budgets[h] - 2
        base = -mag((nb, nb))
        for i in range(nb):
            cand = np.arange(1, i)
            if 0 < want < len(cand):
                base[i, rng.choice(cand, size=want, replace=False)] *= -1.0
        sc[h] = base
    run.select_step(torch.from_numpy(sc.reshape(-1)).to("cuda:0"))
    torch.cuda.synchronize()
    ptr_o, idx_o = orc.select_blocks([sc], wl.budgets)
    np.testing.assert_array_equal(run.sel_ptr_host, ptr_o)
    np.testing.assert_array_equal(run.sel_idx_host(), idx_o)


def test_deterministic_across_runs():
    wl = make_workload(1, seqlens=[2048])
    run = _gpu()(wl).run_all()
    o1, l1, i1 = run.out.clone(), run.lse.clone(), run.sel_idx.clone()
    run.out.zero_(); run.lse.zero_(); run.sel_idx.fill_(-1)
    run.run_all()
    assert torch.equal(run.out.view(torch.int16), o1.view(torch.int16))
    assert torch.equal(run.lse, l1) and torch.equal(run.sel_idx, i1)


def test_rising_and_falling_scores():
    # Keys whose logits climb by several nats from tile to tile (the running reference of the
    # softmax is too low again and again: rescale path), then fall far below it (stale
    # reference, probabilities near the bottom of the fp32 range).  Every block selected.
    from workloads import bf16_bits_from_f32, f32_from_bf16_bits
    wl = make_custom([128 * 14 + 50], 2, 1, 128, [15, 15], seed=91, name="rising")
    q = f32_from_bf16_bits(wl.q)
    k = f32_from_bf16_bits(wl.k)
    u = q[:, 0, :].mean(axis=0)
    u /= np.linalg.norm(u)
    T = k.shape[0]
    tile = np.arange(T) // 64
    push = np.where(tile < 18, 9.0 * tile, 9.0 * 18 - 30.0 * (tile - 18))      # up 18 tiles, then steeply down
    k[:, 0, :] += (push[:, None] * u[None, :]).astype(np.float32)
    wl.k = bf16_bits_from_f32(k)
    full_parity(wl)


def test_budgets_from_max_min_shifting():
    # The producer feeds the consumer: budgets come out of shplb_shift_budgets run on synthetic
    # recovery curves (saturating, head-dependent rate), 8 blocks per head on average, lower bound 2.
    import paper_2603_10353_amd as S
    nb, hq = 40, 8
    rate = np.exp(np.random.default_rng(17).uniform(np.log(0.03), np.log(1.5), size=hq))
    rec = 1.0 - np.exp(-np.outer(rate, np.arange(nb + 1)))
    budgets, moves = S.shplb_shift_budgets(rec, total=8 * hq, lower=2)
    bo, mo = orc.shift_budgets(rec, 8 * hq, 2)
    np.testing.assert_array_equal(budgets, bo)
    assert moves == mo and moves > 0 and budgets.min() >= 2 and budgets.sum() == 8 * hq
    wl = make_custom([128 * nb - 9], hq, 2, 128, budgets.tolist(), seed=93, name="shifted_budgets")
    full_parity(wl)
