"""The attention entry point that allocates nothing (static scratch inside the library) against
the workspace entry point: same kernels, so outputs must agree bit for bit -- on two calls in a
row, the second on a smaller input (the static array then still holds the first call's queues)."""
import numpy as np
import pytest
import torch

import paper_2603_10353_amd as S
from workloads import make_custom, make_workload

pytestmark = pytest.mark.gpu


def _both_ways(wl):
    from harness import DevicePass
    print("case", wl.name, "seqlens", np.diff(wl.cu_seqlens).tolist(), "heads", wl.n_q_heads, wl.n_kv_heads,
          "block", wl.block, flush=True)
    run = DevicePass(wl).run_all()                     # scores, selection, attention through the workspace entry point
    ref_out, ref_lse = run.out.clone(), run.lse.clone()
    ref_stats = run.stats_host().copy()
    run.out.zero_()
    run.lse.zero_()
    run.stats.zero_()
    reserved = torch.cuda.memory_reserved()
    S.shplb_sparse_attn_prefill_static(run.p, run.q, run.k, run.v, run.sel_ptr, run.sel_idx, run.out, run.lse,
                                       run.stats, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert torch.cuda.memory_reserved() == reserved
    assert torch.equal(run.out.view(torch.int16), ref_out.view(torch.int16))
    assert torch.equal(run.lse, ref_lse)
    st = run.stats_host()
    assert st["n_items"].sum() == ref_stats["n_items"].sum() == run.rows
    assert st["cost_blocks"].sum() == ref_stats["cost_blocks"].sum() == run.sel_ptr_host[-1]
    assert bool(ref_out.any())
    return run


def test_static_scratch_matches_workspace_twice_second_smaller():
    # first: 20 480 rows of two sequences (five-launch ordering); second: 288 rows (single-workgroup
    # ordering) with block 64, on whatever the first call left in the array
    rng = np.random.default_rng(7)
    big = make_custom([128 * 400 + 9, 128 * 239 + 100], 32, 8, 128, rng.choice([2, 3, 6, 11, 30, 999], size=64),
                      seed=301, name="static_big")
    _both_ways(big)
    small = make_custom([64 * 35 + 7, 64], 8, 4, 64, [2, 4, 999, 7, 3, 5, 9, 2], seed=302, name="static_small")
    _both_ways(small)
    # and the first size again after the small one
    _both_ways(make_workload(1, seqlens=[128 * 37 + 5]))


def test_static_scratch_refuses_what_does_not_fit():
    # 4096 blocks x 32 heads = 131 072 rows need about 13 MB of scratch: refused on the host, nothing launched
    wl_shape = S.Problem(np.asarray([0, 128 * 4096], np.int32), 32, 8, 128)
    one = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(S.ShplbError) as e:
        S.shplb_sparse_attn_prefill_static(wl_shape, one, one, one, one, one, one, None, None, None)
    assert e.value.status == -4


def test_static_scratch_entry_point_in_a_hip_graph():
    # What the entry point is for: captured into a HIP graph (after one call outside the capture, which
    # looks up the array's address) and replayed with eager work in between; every replay must
    # reproduce the workspace entry point's result bit for bit.
    from harness import DevicePass
    wl = make_workload(1, seqlens=[128 * 29 + 17])
    run = DevicePass(wl).run_all()
    ref_out, ref_lse = run.out.clone(), run.lse.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        S.shplb_sparse_attn_prefill_static(run.p, run.q, run.k, run.v, run.sel_ptr, run.sel_idx, run.out, run.lse,
                                           None, side)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            S.shplb_sparse_attn_prefill_static(run.p, run.q, run.k, run.v, run.sel_ptr, run.sel_idx, run.out,
                                               run.lse, None, side)
    torch.cuda.synchronize()
    for replay in range(3):
        run.out.zero_(); run.lse.zero_()
        run.ws.random_(0, 255)                       # eager work between replays; the workspace is not used
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(run.out.view(torch.int16), ref_out.view(torch.int16)), replay
        assert torch.equal(run.lse, ref_lse), replay
