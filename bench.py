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
SAMPLE_PARITY_MAX_ABS = 2e-2      # attention output against the oracle rows of the CPU sample

PROFILE_DIR = os.path.join(ROOT, "profiles")


def measured_traffic_bytes(workload_name, kernel):
    """HBM bytes of one launch of `kernel` on `workload_name` as rocprofv3 counted them (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a copy of known size): the line `traffic_bytes_per_launch <workload>
    <kernel> <bytes>` that paper_2603_10353_amd/profile_summary.py writes into profiles/.  None when no
    summary holds that pair."""
    try:
        names = sorted(os.listdir(PROFILE_DIR))
    except OSError:
        return None
    for name in names:
        if not name.endswith(".txt"):
            continue
        with open(os.path.join(PROFILE_DIR, name)) as f:
            for line in f:
                w = line.split()
                if len(w) == 4 and w[0] == "traffic_bytes_per_launch" and w[1] == workload_name and w[2] == kernel:
                    return float(w[3])
    return None


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
        if t_used >= budget_s or len(rows) >= 1024:
            break
    rec = dict(value=4.0 * d * pairs / t_used / 1e12, unit="TFLOP/s", cores=int(cores), kind="oracle",
               sample="attention oracle (numpy fp64) on %d seeded (head, query-block) rows incl. the 4 "
                      "costliest, %.1f s" % (len(rows), t_used))
    return rec, outs


class ClockSampler:
    """Shader clock as the driver reports it (rocm-smi), sampled from a thread while the device works."""

    def __init__(self):
        import threading
        self.samples, self.stop = [], False
        self.thread = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import re
        import subprocess
        while not self.stop:
            t = time.perf_counter()
            try:
                out = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True,
                                     timeout=10).stdout
                m = re.search(r"sclk clock speed:\W+(\d+)Mhz", out)
                if m:
                    self.samples.append((t, int(m.group(1))))
            except Exception:
                return
            time.sleep(0.02)

    def __enter__(self):
        self.thread.start()
        return self

    def __exit__(self, *exc):
        self.stop = True
        self.thread.join(timeout=15)

    def median_mhz(self, t0, t1):
        got = sorted(v for (t, v) in self.samples if t0 <= t <= t1)
        return (got[len(got) // 2], len(got)) if got else (None, 0)


class Pass:
    """Device-resident buffers of one workload and the timed loop over whole steps."""

    def __init__(self, S, torch, wl, split_slots=0):
        from paper_2603_10353_amd.binding import WG_STATS_DTYPE
        self.S, self.torch, self.wl, self.split_slots = S, torch, wl, split_slots
        self.stats_dtype = WG_STATS_DTYPE
        dev = "cuda:0"
        to_dev = lambda b: torch.from_numpy(b.view(np.int16)).to(dev).view(torch.bfloat16)
        self.q, self.k, self.v = to_dev(wl.q), to_dev(wl.k), to_dev(wl.v)
        self.p = S.Problem(wl.cu_seqlens, wl.n_q_heads, wl.n_kv_heads, wl.block, wl.head_dim)
        self.rows = S.shplb_num_rows(self.p)
        ws_bytes = S.shplb_split_workspace_bytes(self.p, split_slots) if split_slots else S.shplb_workspace_bytes(self.p)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.scores = torch.empty(int(S.shplb_score_layout(self.p)[-1]), dtype=torch.float32, device=dev)
        self.sel_ptr_h = S.shplb_sel_row_ptr(self.p, wl.budgets)
        self.sel_ptr = torch.from_numpy(self.sel_ptr_h).to(dev)
        self.sel_idx = torch.empty(int(self.sel_ptr_h[-1]), dtype=torch.int32, device=dev)
        self.out = torch.empty_like(self.q)
        self.total_tokens = self.q.shape[0]
        self.lse = torch.empty((wl.n_q_heads, self.total_tokens), dtype=torch.float32, device=dev)
        n_wg = S.shplb_sched_num_workgroups(self.p)
        self.stats = torch.zeros(n_wg * WG_STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
        self.stream = torch.cuda.current_stream()

    def step(self, ev=None):
        S, p, st = self.S, self.p, self.stream
        if ev:
            ev[0].record()
        S.shplb_block_scores(p, self.q, self.k, self.scores, self.ws, st)
        if ev:
            ev[1].record()
        S.shplb_select_topk_per_head(p, self.scores, self.wl.budgets, self.sel_ptr, self.sel_idx, st)
        if ev:
            ev[2].record()
        if self.split_slots:
            S.shplb_sparse_attn_prefill_split(p, self.q, self.k, self.v, self.sel_ptr, self.sel_idx, self.out,
                                              self.lse, self.stats, self.ws, self.split_slots, st)
        else:
            S.shplb_sparse_attn_prefill(p, self.q, self.k, self.v, self.sel_ptr, self.sel_idx, self.out,
                                        self.lse, self.stats, self.ws, st)
        if ev:
            ev[3].record()

    def measure(self, steps, warmup):
        """warmup untimed steps, then exactly `steps` timed ones between two synchronisations.
        Phase times come from HIP events recorded on the stream the kernels are launched on."""
        torch, wl = self.torch, self.wl
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        t0 = time.perf_counter()
        for it in range(steps):
            self.step(events[it])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_per_step = wall * 1e3 / steps
        ph = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in events])
        score_ms, select_ms, attn_ms = [float(x) for x in ph.mean(axis=0)]
        pairs = selected_pairs(wl.cu_seqlens, wl.block, wl.n_q_heads, self.sel_ptr_h)
        flops = 4.0 * wl.head_dim * pairs
        tri = 4 * wl.n_q_heads * sum(nb * (nb + 1) // 2 for nb in wl.n_blocks)
        score_bytes = (wl.n_q_heads + wl.n_kv_heads) * self.total_tokens * wl.head_dim * 2 + tri
        select_bytes = tri + 4 * int(self.sel_ptr_h[-1])
        st = np.frombuffer(self.stats.cpu().numpy().tobytes(), dtype=self.stats_dtype)
        busy = (st["t_last"] - st["t_first"]).astype(np.float64)
        active = st["n_items"] > 0
        imb_time = float(busy[active].max() / busy[active].mean() - 1.0) if active.any() else None
        cost = st["cost_blocks"].astype(np.float64)
        span = float(st["t_last"][active].max() - st["t_first"][active].min())
        kernel = "attn_pipe_kernel"
        attn_tflops = flops / (attn_ms * 1e-3) / 1e12
        return {
            "ms_per_step": ms_per_step, "value": flops / (ms_per_step * 1e-3) / 1e12,
            "pairs": int(pairs), "flops": flops,
            "phases_ms": {"block_scores": score_ms, "select_topk": select_ms, "sparse_attn": attn_ms},
            "score_hbm_gbps": score_bytes / (score_ms * 1e-3) / 1e9,
            "score_hbm_frac": score_bytes / (score_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "select_hbm_gbps": select_bytes / (select_ms * 1e-3) / 1e9,
            "cu_imbalance": {"busy_time_max_over_mean_minus_1": imb_time,
                             "cost_max_over_mean_minus_1": float(cost.max() / cost.mean() - 1.0),
                             "idle_fraction_of_span": float(1.0 - busy[active].sum() / (span * len(st))),
                             "workgroups": int(len(st))},
            "roofline": {"bound": "mfma", "achieved": attn_tflops, "peak": BF16_MFMA_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": attn_tflops / BF16_MFMA_PEAK_TFLOPS,
                         "traffic": measured_traffic_bytes(wl.name, kernel), "kernel": kernel, "kernel_ms": attn_ms},
        }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-32k", action="store_true",
                    help="skip the second, short measurement of the 32K layer (workload cfg1), the other "
                         "context length the metric names; it is only made when the main workload is cfg2")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the two short MFMA-only launches that measure what the matrix pipe sustains")
    ap.add_argument("--profile-pass", action="store_true",
                    help="also time the offline recovery profiles (shplb_block_mass, shplb_token_recovery: dense passes; "
                         "not part of a step)")
    ap.add_argument("--split-slots", type=int, default=0,
                    help="run the attention step through shplb_sparse_attn_prefill_split with this many "
                         "partial-result slots (long rows cut along the keys); 0 = whole rows")
    ap.add_argument("--sample-clocks", action="store_true",
                    help="sample the shader clock (rocm-smi) from a thread during the timed steps and report its "
                         "median as sclk_during_timed_steps; use with enough --steps to last a few seconds")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run one plain 1 GiB elementwise copy kernel (reference for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build covers one GPU's share of the path; run with --gpus 1 "
                 "(heads shard across GPUs with no exchange; nothing here needs a second GPU)")

    import torch
    import paper_2603_10353_amd as S
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
    run = Pass(S, torch, wl, args.split_slots)
    stream = run.stream

    if args.traffic_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if args.sample_clocks:
        with ClockSampler() as clocks:
            t0 = time.perf_counter()
            m = run.measure(args.steps, args.warmup)
            t1 = time.perf_counter()
        # samples from the timed steps only (the warm-up comes first; leave it a margin)
        mhz, n = clocks.median_mhz(t1 - 0.9 * args.steps * m["ms_per_step"] * 1e-3, t1)
        m["sclk"] = {"median_mhz": mhz, "samples": n, "source": "rocm-smi --showclocks during the timed steps"}
    else:
        m = run.measure(args.steps, args.warmup)
    attn_tflops = m["roofline"]["achieved"]

    result = {
        "metric": "effective TFLOP/s on selected blocks (per-layer prefill latency = ms_per_step; 128K here, "
                  "32K under latency_32k_ms)",
        "value": m["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "seqlens": [int(x) for x in np.diff(wl.cu_seqlens)],
                   "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim,
                   "block": wl.block, "rows": int(run.rows), "selected_blocks": int(run.sel_ptr_h[-1]),
                   "selected_pairs": m["pairs"], "selected_flops": m["flops"], "seed": wl.seed, **extra},
        "phases_ms": m["phases_ms"],
        "score_hbm_gbps": m["score_hbm_gbps"], "score_hbm_frac": m["score_hbm_frac"],
        "select_hbm_gbps": m["select_hbm_gbps"],
        "cu_imbalance": m["cu_imbalance"],
        "roofline": m["roofline"],
        "host_input_generation_s": t_gen,
    }
    if "sclk" in m:
        result["sclk_during_timed_steps"] = m["sclk"]

    if cfg == 2 and not args.no_32k:
        # The metric names two context lengths.  The 32K layer (workload cfg1) is measured the same
        # way, in the same process, after the main workload's timed region.
        wl32 = make_workload(1)
        run32 = Pass(S, torch, wl32)
        # the card idles while the host draws this layer's inputs, and a 2 ms step does not bring the clock
        # back by itself: at least 50 untimed steps (0.1 s) first, so that the timed ones run at the clock a
        # stream of such layers sees (measured on one box: 2.017 ms after 3 untimed steps, 1.956 after 20,
        # 1.936 after 60)
        m32 = run32.measure(args.steps, max(args.warmup, 50))
        result["warmup_32k"] = max(args.warmup, 50)
        result["latency_32k_ms"] = m32["ms_per_step"]
        result["tflops_32k"] = m32["value"]
        result["workload_32k"] = wl32.name
        result["phases_32k_ms"] = m32["phases_ms"]
        result["roofline_32k"] = m32["roofline"]
        result["score_hbm_frac_32k"] = m32["score_hbm_frac"]
        result["cu_imbalance_32k"] = m32["cu_imbalance"]
        del run32, wl32

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
        mass = torch.empty_like(run.scores)
        S.shplb_block_mass(run.p, run.q, run.k, mass, stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            S.shplb_block_mass(run.p, run.q, run.k, mass, stream)
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
        # the same ratio at token granularity, at the budget Section 2.4 profiles (k = 4096 tokens)
        rec = torch.empty((1, wl.n_q_heads, int(wl.cu_seqlens[-1])), dtype=torch.float32, device="cuda:0")
        S.shplb_token_recovery(run.p, run.q, run.k, [4096], rec, stream)
        torch.cuda.synchronize()
        e0.record()
        S.shplb_token_recovery(run.p, run.q, run.k, [4096], rec, stream)
        e1.record()
        torch.cuda.synchronize()
        heads = S.shplb_token_recovery_heads(run.p, rec.cpu().numpy())
        result["profile_pass"]["token_recovery_k4096"] = {
            "kernel": "token_recovery_kernel", "ms": e0.elapsed_time(e1),
            "recovery_per_head_min_max": [float(heads.min()), float(heads.max())]}
        del rec

    if not args.no_cpu_baseline:
        idx_h = run.sel_idx.cpu().numpy()
        rec, outs = cpu_baseline(wl, run.sel_ptr_h, idx_h)
        result["cpu_baseline"] = rec
        out_h = run.out.to(torch.float32).cpu().numpy()
        worst, worst_row = 0.0, None
        for r, (s, h, i, o, _l) in outs.items():
            t_begin = int(wl.cu_seqlens[s]) + i * wl.block
            d = float(np.abs(out_h[t_begin:t_begin + o.shape[0], h, :] - o).max())
            if not d <= worst:                      # also catches NaN
                worst, worst_row = d, (r, s, h, i)
        result["sample_parity_max_abs"] = worst
        if not worst <= SAMPLE_PARITY_MAX_ABS:
            print(json.dumps(result))
            sys.exit("bench.py: attention output differs from the oracle by %.4g (> %.3g) on row %d "
                     "(sequence %d, head %d, query block %d): the throughput above is not valid"
                     % ((worst, SAMPLE_PARITY_MAX_ABS) + worst_row))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
