#!/usr/bin/env python3
"""Benchmark of the S-HPLB hot path on one MI355X.

A step = one pass of the whole path over one synthetic layer input already resident
in HBM: shplb_block_scores -> shplb_select_topk_per_head -> shplb_sparse_attn_prefill
(which orders the work items and runs the persistent attention kernel).

Metric: effective TFLOP/s on the selected blocks = 4 * head_dim * (unmasked
query-key pairs inside selected blocks) / step time; the per-layer prefill latency
is ms_per_step.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {"cfg0": 0, "cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4}
BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
HBM_PEAK_GBPS = 8000.0

# HBM traffic of one attention launch measured with rocprofv3 --pmc (FETCH_SIZE, then
# WRITE_SIZE), scaled by a copy kernel of known size; see profiles/.  None = not measured.
MEASURED_TRAFFIC_BYTES = {"cfg2_llama3_8b_128k": 2 * 13371986.6 * 1024 + 1072592.9 * 1024}


def selected_pairs(cu_seqlens, block, n_q_heads, sel_ptr_host):
    """Unmasked (query token, key token) pairs inside the selected blocks.  Every
    selected block other than the diagonal one is full and fully visible; the diagonal
    block contributes cnt*(cnt+1)/2 for its cnt valid tokens."""
    total = 0
    r = 0
    counts = np.diff(sel_ptr_host)
    for s in range(len(cu_seqlens) - 1):
        length = int(cu_seqlens[s + 1] - cu_seqlens[s])
        nb = -(-length // block)
        cnt = np.full(nb, block, np.int64)
        cnt[-1] = length - (nb - 1) * block
        for _h in range(n_q_heads):
            n = counts[r:r + nb].astype(np.int64)
            total += int(((n - 1) * cnt * block + cnt * (cnt + 1) // 2).sum())
            r += nb
    return total


def pick_config3_heads(S):
    """Config 3: the layer's 16 KV groups are dealt to 8 parts of 2 groups each by
    shplb_balance_heads on their causal block cost; the bench runs the heaviest part."""
    from workloads import CONFIGS, layer_budgets
    cfg = CONFIGS[3]
    lb = layer_budgets(3)
    nb = lb["n_blocks"][0]
    k = np.clip(lb["budgets"][0].astype(np.int64), 2, nb)
    head_cost = k * nb - k * (k - 1) // 2
    g = cfg["n_q_heads"] // cfg["n_kv_heads"]
    group_cost = head_cost.reshape(-1, g).sum(axis=1)
    part, loads = S.shplb_balance_heads(group_cost, cfg["n_parts"], cfg["groups_per_part"])
    heavy = int(np.argmax(loads))
    groups = [x for x in range(len(group_cost)) if part[x] == heavy]
    heads = [gg * g + j for gg in groups for j in range(g)]
    return heads, loads


def cpu_baseline(wl, sel_ptr, sel_idx, budget_s=15.0):
    """The oracle as it stands, timed on the host cores on a bounded row sample:
    seeded (head, query block) rows, costliest first, until about budget_s of CPU work.
    Returns the baseline record and the rows (for a spot parity check)."""
    from oracle import shplb_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    counts = np.diff(sel_ptr)
    rng = np.random.default_rng(12345)
    heavy = np.argsort(-counts, kind="stable")[:4]
    rest = rng.permutation(len(counts))
    rows, pairs, t_used = [], 0, 0.0
    outs = {}
    d, blk = wl.head_dim, wl.block
    for r in list(heavy) + list(rest):
        r = int(r)
        if r in outs:
            continue
        s, h, i = orc.row_decode(wl.cu_seqlens, blk, wl.n_q_heads, r)
        sel = sel_idx[sel_ptr[r]:sel_ptr[r + 1]]
        t0 = time.perf_counter()
        o, lse = orc.sparse_attention_row(wl.q, wl.k, wl.v, wl.cu_seqlens, blk, s, h, i, sel)
        t_used += time.perf_counter() - t0
        outs[r] = (s, h, i, o, lse)
        nq = o.shape[0]
        pairs += (len(sel) - 1) * nq * blk + nq * (nq + 1) // 2
        rows.append(r)
        if t_used >= budget_s or len(rows) >= 512:
            break
    rec = dict(value=4.0 * d * pairs / t_used / 1e12, unit="TFLOP/s", cores=int(cores), kind="oracle",
               sample="attention oracle (numpy fp64) on %d seeded (head, query-block) rows incl. the 4 "
                      "costliest, %.1f s" % (len(rows), t_used))
    return rec, outs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the two short MFMA-only launches that measure what the matrix pipe sustains")
    ap.add_argument("--profile-pass", action="store_true",
                    help="also time the offline recovery profile (shplb_block_mass, a dense pass; not part of a step)")
    ap.add_argument("--split-slots", type=int, default=0,
                    help="run the attention step through shplb_sparse_attn_prefill_split with this many "
                         "partial-result slots (long rows cut along the keys; block 128 only); 0 = whole rows")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run one plain 1 GiB elementwise copy kernel (reference for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build covers one GPU's share of the path; run with --gpus 1 "
                 "(heads shard across GPUs with no exchange; nothing here needs a second GPU)")

    import torch
    import paper_2603_10353_amd as S
    from paper_2603_10353_amd.binding import WG_STATS_DTYPE
    if not os.path.exists(S.lib_path()):
        from paper_2603_10353_amd.build import build
        build(verbose=False)
    from workloads import make_workload

    cfg = WORKLOADS[args.workload]
    t_gen = time.perf_counter()
    extra = {}
    if args.split_slots:
        extra["split_slots"] = args.split_slots
    if cfg == 3:
        heads, loads = pick_config3_heads(S)
        wl = make_workload(3, q_heads=heads)
        extra["partition_loads"] = [int(x) for x in loads]
        extra["layer_heads"] = heads
    else:
        wl = make_workload(cfg)
    t_gen = time.perf_counter() - t_gen

    dev = "cuda:0"
    torch.cuda.set_device(0)
    to_dev = lambda b: torch.from_numpy(b.view(np.int16)).to(dev).view(torch.bfloat16)
    q, k, v = to_dev(wl.q), to_dev(wl.k), to_dev(wl.v)
    p = S.Problem(wl.cu_seqlens, wl.n_q_heads, wl.n_kv_heads, wl.block, wl.head_dim)
    rows = S.shplb_num_rows(p)
    ws_bytes = S.shplb_split_workspace_bytes(p, args.split_slots) if args.split_slots else S.shplb_workspace_bytes(p)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    score_off = S.shplb_score_layout(p)
    scores = torch.empty(int(score_off[-1]), dtype=torch.float32, device=dev)
    sel_ptr_h = S.shplb_sel_row_ptr(p, wl.budgets)
    sel_ptr = torch.from_numpy(sel_ptr_h).to(dev)
    sel_idx = torch.empty(int(sel_ptr_h[-1]), dtype=torch.int32, device=dev)
    out = torch.empty_like(q)
    total_tokens = q.shape[0]
    lse = torch.empty((wl.n_q_heads, total_tokens), dtype=torch.float32, device=dev)
    n_wg = S.shplb_sched_num_workgroups(p)
    stats = torch.zeros(n_wg * WG_STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(ev=None):
        if ev:
            ev[0].record()
        S.shplb_block_scores(p, q, k, scores, ws, stream)
        if ev:
            ev[1].record()
        S.shplb_select_topk_per_head(p, scores, wl.budgets, sel_ptr, sel_idx, stream)
        if ev:
            ev[2].record()
        if args.split_slots:
            S.shplb_sparse_attn_prefill_split(p, q, k, v, sel_ptr, sel_idx, out, lse, stats, ws, args.split_slots,
                                              stream)
        else:
            S.shplb_sparse_attn_prefill(p, q, k, v, sel_ptr, sel_idx, out, lse, stats, ws, stream)
        if ev:
            ev[3].record()

    if args.traffic_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for it in range(args.steps):
        step(events[it])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    ph = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in events])
    score_ms, select_ms, attn_ms = [float(x) for x in ph.mean(axis=0)]

    pairs = selected_pairs(wl.cu_seqlens, wl.block, wl.n_q_heads, sel_ptr_h)
    flops = 4.0 * wl.head_dim * pairs
    value = flops / (ms_per_step * 1e-3) / 1e12
    attn_tflops = flops / (attn_ms * 1e-3) / 1e12

    nbs = wl.n_blocks
    score_bytes = (wl.n_q_heads + wl.n_kv_heads) * total_tokens * wl.head_dim * 2 \
        + 4 * wl.n_q_heads * sum(nb * (nb + 1) // 2 for nb in nbs)
    select_bytes = 4 * wl.n_q_heads * sum(nb * (nb + 1) // 2 for nb in nbs) + 4 * int(sel_ptr_h[-1])

    st = np.frombuffer(stats.cpu().numpy().tobytes(), dtype=WG_STATS_DTYPE)
    busy = (st["t_last"] - st["t_first"]).astype(np.float64)
    active = st["n_items"] > 0
    imb_time = float(busy[active].max() / busy[active].mean() - 1.0) if active.any() else None
    cost = st["cost_blocks"].astype(np.float64)
    imb_cost = float(cost.max() / cost.mean() - 1.0)
    span = float(st["t_last"][active].max() - st["t_first"][active].min())
    idle_frac = float(1.0 - busy[active].sum() / (span * len(st)))

    result = {
        "metric": "effective TFLOP/s on selected blocks (per-layer prefill latency = ms_per_step)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "seqlens": [int(x) for x in np.diff(wl.cu_seqlens)],
                   "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim,
                   "block": wl.block, "rows": int(rows), "selected_blocks": int(sel_ptr_h[-1]),
                   "selected_pairs": int(pairs), "selected_flops": flops, "seed": wl.seed, **extra},
        "phases_ms": {"block_scores": score_ms, "select_topk": select_ms, "sparse_attn": attn_ms},
        "score_hbm_gbps": score_bytes / (score_ms * 1e-3) / 1e9,
        "score_hbm_frac": score_bytes / (score_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "select_hbm_gbps": select_bytes / (select_ms * 1e-3) / 1e9,
        "cu_imbalance": {"busy_time_max_over_mean_minus_1": imb_time, "cost_max_over_mean_minus_1": imb_cost,
                         "idle_fraction_of_span": idle_frac, "workgroups": int(len(st))},
        "roofline": {"bound": "mfma", "achieved": attn_tflops, "peak": BF16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": attn_tflops / BF16_MFMA_PEAK_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name), "kernel": "attn_pipe_kernel" if wl.block == 128 else "attn_kernel",
                     "kernel_ms": attn_ms},
        "host_input_generation_s": t_gen,
    }

    if not args.no_mfma_ceiling:
        # What the bf16 matrix pipe sustains on this chip with nothing else going on: the published
        # peak is the roofline's denominator, this is the ceiling a kernel can actually approach.
        n_probe, iters = 1024, 120000            # 0.13-0.17 s per launch: long enough for the clock to settle
        scratch = torch.zeros(16 + n_probe * 2048, dtype=torch.uint8, device=dev)
        ceiling = {}
        for name, rnd in (("constant_operands", False), ("random_operands", True)):
            S.shplb_probe_mfma_rate(rnd, iters // 4, n_probe, scratch, stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            S.shplb_probe_mfma_rate(rnd, iters, n_probe, scratch, stream)
            e1.record()
            torch.cuda.synchronize()
            clk = scratch[:16].cpu().numpy().view(np.uint64)
            ceiling[name] = {"tflops": n_probe * 8 * 8 * iters * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12,
                             "clock_mhz": float(clk[0]) / (float(clk[1]) * 0.01)}
        ceiling["attention_frac_of_random_operand_rate"] = attn_tflops / ceiling["random_operands"]["tflops"]
        result["mfma_ceiling"] = ceiling
        del scratch

    if args.profile_pass:
        mass = torch.empty_like(scores)
        S.shplb_block_mass(p, q, k, mass, stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            S.shplb_block_mass(p, q, k, mass, stream)
        e1.record()
        torch.cuda.synchronize()
        mass_ms = e0.elapsed_time(e1) / 3
        causal_pairs = sum(int(n) * (int(n) + 1) // 2 for n in np.diff(wl.cu_seqlens)) * wl.n_q_heads
        # one QK^T over the causal triangle is what the profile needs; the kernel runs it twice
        # (softmax statistics, then probabilities)
        result["profile_pass"] = {"kernel": "mass_kernel", "ms": mass_ms,
                                  "tflops_one_qk_pass": 2.0 * wl.head_dim * causal_pairs / (mass_ms * 1e-3) / 1e12,
                                  "frac_of_bf16_mfma_peak_executed": 2 * 2.0 * wl.head_dim * causal_pairs
                                  / (mass_ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
        del mass

    if not args.no_cpu_baseline:
        idx_h = sel_idx.cpu().numpy()
        rec, outs = cpu_baseline(wl, sel_ptr_h, idx_h)
        result["cpu_baseline"] = rec
        out_h = out.to(torch.float32).cpu().numpy()
        worst = 0.0
        for r, (s, h, i, o, _l) in outs.items():
            t_begin = int(wl.cu_seqlens[s]) + i * wl.block
            worst = max(worst, float(np.abs(out_h[t_begin:t_begin + o.shape[0], h, :] - o).max()))
        result["sample_parity_max_abs"] = worst
    print(json.dumps(result))


if __name__ == "__main__":
    main()
