#!/usr/bin/env python3
"""Head-parallel load balancer, with and without (the paper's ablation, Section 5, Ablation Study).

The paper measures attention latency of a head-parallel layer over parallelism degrees at 128K and
over context lengths at degree 4, with heads assigned to GPUs in order ("naive") and by its greedy
balancer.  One GPU can show the same thing part by part: a layer's latency under head parallelism is
the latency of its slowest part (parts exchange nothing until the barrier behind attention), so
every part's share is run on this GPU through the whole hot path and the maximum is taken.

Units of the assignment are query heads, as in Section 3.3: cost of a head = its causal block cost
under the layer's budgets; "naive" gives every part the same number of consecutive heads, "greedy"
is shplb_balance_heads (parts may end up with different head counts).  A part's share is run with
the distinct KV heads its query heads need, shared among them as in the layer (an explicit query-head
to KV-head map, since a part's groups need not be whole).  Inputs
are the synthetic 128K layer of the benchmark (workload cfg2) and shorter contexts of the same
recipe.  Prints one table; `--json` adds one JSON line per row.

    python balance_ablation.py [--steps 3] [--warmup 1] [--json]
"""
import argparse
import json
import sys
import time

import numpy as np


def head_costs(budgets, nb):
    k = np.clip(budgets.astype(np.int64), 2, nb)
    return k * nb - k * (k - 1) // 2                 # selected blocks over all causal rows of a head


def share_of(layer, heads):
    """The part of a layer's workload that a GPU holding `heads` works on: those query heads and the
    distinct KV heads they read, each held once (the part's query heads share them as in the layer)."""
    from workloads import take_heads
    return take_heads(layer, heads)


def run_share(S, torch, wl, steps, warmup):
    """ms per pass of the whole hot path over one part's heads."""
    from paper_2603_10353_amd.binding import WG_STATS_DTYPE
    dev = "cuda:0"
    to_dev = lambda b: torch.from_numpy(b.view(np.int16)).to(dev).view(torch.bfloat16)
    q, k, v = to_dev(wl.q), to_dev(wl.k), to_dev(wl.v)
    p = S.Problem(wl.cu_seqlens, wl.n_q_heads, wl.n_kv_heads, wl.block, wl.head_dim, kv_head_of=wl.kv_head_of)
    ws = torch.empty(S.shplb_workspace_bytes(p), dtype=torch.uint8, device=dev)
    scores = torch.empty(int(S.shplb_score_layout(p)[-1]), dtype=torch.float32, device=dev)
    sel_ptr_h = S.shplb_sel_row_ptr(p, wl.budgets)
    sel_ptr = torch.from_numpy(sel_ptr_h).to(dev)
    sel_idx = torch.empty(int(sel_ptr_h[-1]), dtype=torch.int32, device=dev)
    out = torch.empty_like(q)
    lse = torch.empty((wl.n_q_heads, q.shape[0]), dtype=torch.float32, device=dev)
    stats = torch.zeros(S.shplb_sched_num_workgroups(p) * WG_STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        S.shplb_block_scores(p, q, k, scores, ws, stream)
        S.shplb_select_topk_per_head(p, scores, wl.budgets, sel_ptr, sel_idx, stream)
        S.shplb_sparse_attn_prefill(p, q, k, v, sel_ptr, sel_idx, out, lse, stats, ws, stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def ablation_case(S, seqlen, degree, n_heads, part_ms):
    """One row of the ablation: consecutive heads against shplb_balance_heads for one context length and
    parallelism degree.  part_ms(seqlen, heads) -> ms of the whole hot path over that part's share."""
    from workloads import layer_budgets
    lb = layer_budgets(2, [seqlen])
    cost = head_costs(lb["budgets"][0], lb["n_blocks"][0])
    per = n_heads // degree
    naive = [list(range(d * per, (d + 1) * per)) for d in range(degree)]
    part_of, _ = S.shplb_balance_heads(cost, degree)
    greedy = [[x for x in range(n_heads) if part_of[x] == d] for d in range(degree)]
    rec = {"tokens": seqlen, "degree": degree}
    for name, parts in (("naive", naive), ("greedy", greedy)):
        loads = [int(cost[p].sum()) for p in parts]
        ms = [part_ms(seqlen, p) for p in parts]
        rec[name] = {"parts": parts, "cost_imbalance": max(loads) / (sum(loads) / degree),
                     "part_ms": ms, "layer_ms": max(ms)}
    rec["speedup"] = rec["naive"]["layer_ms"] / rec["greedy"]["layer_ms"]
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()

    import torch
    import paper_2603_10353_amd as S
    from workloads import CONFIGS, make_workload
    torch.cuda.set_device(0)

    n_heads = CONFIGS[2]["n_q_heads"]
    cases = [(131072, d) for d in (2, 4, 8)] + [(s, 4) for s in (32768, 65536)]
    layers, latency = {}, {}                         # seqlen -> workload; (seqlen, heads of the part) -> ms

    def part_ms(seqlen, heads):
        key = (seqlen, tuple(heads))
        if key not in latency:
            if seqlen not in layers:
                layers.clear()                       # one layer in host memory at a time
                layers[seqlen] = make_workload(2, seqlens=[seqlen])
            latency[key] = run_share(S, torch, share_of(layers[seqlen], heads), args.steps, args.warmup)
            print("  ran %6d tokens, heads %s: %.3f ms" % (seqlen, list(heads), latency[key]), file=sys.stderr,
                  flush=True)
        return latency[key]

    rows = [ablation_case(S, seqlen, degree, n_heads, part_ms) for seqlen, degree in sorted(cases)]

    print("%8s %6s | %-22s | %-22s | %s" % ("tokens", "degree", "naive: I(cost)  ms", "greedy: I(cost)  ms", "naive/greedy"))
    for r in rows:
        print("%8d %6d | %10.3f %10.3f | %10.3f %10.3f | %8.3fx" % (
            r["tokens"], r["degree"], r["naive"]["cost_imbalance"], r["naive"]["layer_ms"],
            r["greedy"]["cost_imbalance"], r["greedy"]["layer_ms"], r["speedup"]))
    if args.json:
        for r in rows:
            print(json.dumps(r))


if __name__ == "__main__":
    main()
