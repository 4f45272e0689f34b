"""The load-balancer ablation (Section 3.3, Eq. 2; Section 5, Ablation Study) at reduced size:
a 32-head synthetic layer at 64K tokens over 4 parts, consecutive heads against
shplb_balance_heads.  (At 16K a part's pass takes 0.4 ms and per-row fixed costs, which the
cost model of Eq. 2 does not see, decide: the balanced parts then measure 6% slower than the
worst consecutive one.  From 32K on the selected blocks dominate.)
Checks what the emulation rests on: a part's share is the part's query heads with the KV
heads they read shared among them, its output equals the oracle's, and where
Eq. 2 says the two assignments differ clearly, the measured latency of the slowest part does too."""
import numpy as np
import pytest
import torch

from oracle import shplb_oracle as orc
from workloads import CONFIGS, make_workload, one_kv_head_per_query_head

from checks import compare_output

pytestmark = pytest.mark.gpu

SEQLEN, DEGREE = 65536, 4


def test_greedy_parts_are_real_shares_and_not_slower_than_consecutive_heads():
    import paper_2603_10353_amd as S
    import balance_ablation as ab
    from harness import DevicePass

    layer = make_workload(2, seqlens=[SEQLEN])
    n_heads = CONFIGS[2]["n_q_heads"]
    latency = {}

    def part_ms(seqlen, heads):
        key = tuple(heads)
        if key not in latency:
            latency[key] = min(ab.run_share(S, torch, ab.share_of(layer, heads), steps=5, warmup=2) for _ in range(2))
        return latency[key]

    rec = ab.ablation_case(S, SEQLEN, DEGREE, n_heads, part_ms)
    print("  naive  I(cost) %.3f  parts ms %s" % (rec["naive"]["cost_imbalance"], np.round(rec["naive"]["part_ms"], 4)))
    print("  greedy I(cost) %.3f  parts ms %s  heads %s" % (rec["greedy"]["cost_imbalance"],
                                                           np.round(rec["greedy"]["part_ms"], 4), rec["greedy"]["parts"]),
          flush=True)

    # the parts cover the layer's heads, each once (Eq. 2's constraints), and greedy balances the cost
    for name in ("naive", "greedy"):
        assert sorted(h for p in rec[name]["parts"] for h in p) == list(range(n_heads))
    assert rec["greedy"]["cost_imbalance"] <= rec["naive"]["cost_imbalance"]

    # a greedy part as a share: distinct KV heads held once, groups of unequal size
    part = max(rec["greedy"]["parts"], key=len)
    share = ab.share_of(layer, part)
    g = layer.n_q_heads // layer.n_kv_heads
    assert share.n_kv_heads == len({h // g for h in part}) and share.n_q_heads == len(part)
    run = DevicePass(share).run_all()
    counts = np.diff(run.sel_ptr_host)
    rows = set(np.argsort(-counts, kind="stable")[:2].tolist())
    rows |= set(np.random.default_rng(3).choice(len(counts), size=24, replace=False).tolist())
    flat = one_kv_head_per_query_head(share)
    out_o, lse_o = orc.sparse_attention(flat.q, flat.k, flat.v, flat.cu_seqlens, flat.block, run.sel_ptr_host,
                                        run.sel_idx_host(), None, rows)
    wa, wr, wl_ = compare_output(run.out_host(), out_o, run.lse_host(), lse_o)
    print("  part %s on %d sampled rows: max abs %.3g max rel %.3g lse %.3g" % (part, len(rows), wa, wr, wl_), flush=True)

    # measured latency follows the cost model where the cost model is clear about it
    if rec["naive"]["cost_imbalance"] > 1.10 * rec["greedy"]["cost_imbalance"]:
        assert rec["greedy"]["layer_ms"] <= 1.02 * rec["naive"]["layer_ms"], rec
