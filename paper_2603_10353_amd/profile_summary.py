"""Turn rocprofv3 output of bench.py runs into the short text summaries kept under profiles/.

Four kinds of runs feed one summary (each optional; run from the repository root, after
`cd /tmp && export TMPDIR=/tmp && cd <repo>`; WL = bench.py's --workload, e.g. cfg2):

  kernel durations   rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/kt_WL -o kt --
                         python3 bench.py --workload WL --steps 5 --warmup 2 --no-cpu-baseline --no-32k
                         > gpurun_out/kt_WL.log
  HBM reads          rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/pmc_fetch_WL -o pmc --
                         python3 bench.py --workload WL --steps 2 --warmup 1 --no-cpu-baseline --no-32k
                         --no-mfma-ceiling --traffic-calibration
  HBM writes         the same with WRITE_SIZE into gpurun_out/pmc_write_WL
  SQ counters        the same with up to eight SQ_ counters per run into gpurun_out/pmc_sq<x>_WL
                         (without --traffic-calibration)

    python3 -m paper_2603_10353_amd.profile_summary --workload WL --warmup 2 --out profiles/<name>.txt

Durations are averaged over the timed launches only: the first `--warmup` launches of every
kernel are dropped (bench.py's untimed steps), so a kernel's average can be held against
the step time bench.py printed in the same run.  FETCH_SIZE / WRITE_SIZE readings (KiB per
dispatch) are scaled by what the same counter reads for bench.py's 1 GiB copy kernel; the
line `traffic_bytes_per_launch <workload> <kernel> <bytes>` is what bench.py reports as
roofline.traffic.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

GIB_KIB = float(1 << 20)


def short_name(name: str) -> str:
    m = re.search(r"(\w+)(<[^>]*>)?\(", name)
    if "AUnaryFunctor" in name or "MulFunctor" in name or "BUnaryFunctor" in name:
        return "copy_1GiB"
    return (m.group(1) + (m.group(2) or "")) if m else name[:48]


def find(dirname: str, suffix: str):
    hits = sorted(glob.glob(os.path.join(dirname, "**", "*" + suffix), recursive=True))
    return hits[-1] if hits else None


def kernel_durations(dirname: str, warmup: int):
    """{kernel: [durations in ns of its launches after the first `warmup`]} in dispatch order."""
    path = find(dirname, "_kernel_trace.csv")
    if not path:
        return None
    per = collections.OrderedDict()
    rows = sorted(csv.DictReader(open(path)), key=lambda r: int(r["Start_Timestamp"]))
    for r in rows:
        per.setdefault(short_name(r["Kernel_Name"]), []).append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return {k: v[warmup:] if len(v) > warmup and k.split("<")[0].endswith("_kernel") else v for k, v in per.items()}


def counter_means(dirname: str):
    """{counter: {kernel: (n, mean)}} of one --pmc run."""
    path = find(dirname, "_counter_collection.csv")
    if not path:
        return None
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        agg[r["Counter_Name"]][short_name(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {c: {k: (len(v), sum(v) / len(v)) for k, v in per.items()} for c, per in agg.items()}


def last_json_line(path: str):
    try:
        lines = [l for l in open(path) if l.startswith("{")]
    except OSError:
        return None
    return json.loads(lines[-1]) if lines else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True, help="bench.py --workload value the runs were made with")
    ap.add_argument("--warmup", type=int, default=2, help="--warmup of the kernel-trace run")
    ap.add_argument("--dir", default="gpurun_out", help="where the rocprofv3 output directories are")
    ap.add_argument("--kernel", default="attn_pipe_kernel<128>", help="dominant kernel (traffic line, SQ counters)")
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    wl, d = args.workload, args.dir
    out = []
    bench = last_json_line(os.path.join(d, "kt_%s.log" % wl))
    wl_name = bench["config"]["workload"] if bench else wl
    out.append("# rocprofv3 summary: whole hot path, workload %s (bench.py --workload %s)" % (wl_name, wl))
    out.append("# written by: python3 -m paper_2603_10353_amd.profile_summary --workload %s --warmup %d --out %s"
               % (wl, args.warmup, args.out))

    dur = kernel_durations(os.path.join(d, "kt_" + wl), args.warmup)
    if dur:
        out.append("")
        out.append("Kernel durations, timed launches only (the first %d launches of each library kernel are warm-up)" % args.warmup)
        out.append("  command: rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/kt_%s -o kt -- python3 bench.py "
                   "--workload %s --steps 5 --warmup %d --no-cpu-baseline --no-32k" % (wl, wl, args.warmup))
        out.append("  %-28s %6s %14s %14s %14s" % ("kernel", "calls", "avg_ns", "min_ns", "max_ns"))
        for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
            if v:
                out.append("  %-28s %6d %14.0f %14d %14d" % (k, len(v), sum(v) / len(v), min(v), max(v)))
        if bench:
            out.append("  bench.py line of the same run (HIP events inside bench.py):")
            out.append("    ms_per_step = %.4f" % bench["ms_per_step"])
            out.append("    phases_ms = %s" % json.dumps(bench["phases_ms"]))
            out.append("    roofline = %s" % json.dumps(bench["roofline"]))
            path_kernels = [k for k in dur if k.split("<")[0].endswith("_kernel") and not k.startswith("mfma_rate")]
            total = sum(sum(dur[k]) / len(dur[k]) for k in path_kernels if dur[k])
            out.append("    sum of the path's kernel averages = %.4f ms (<= ms_per_step: launch gaps are the rest)" % (total / 1e6))

    fetch = counter_means(os.path.join(d, "pmc_fetch_" + wl))
    write = counter_means(os.path.join(d, "pmc_write_" + wl))
    if fetch and write:
        f, w = fetch["FETCH_SIZE"], write["WRITE_SIZE"]
        out.append("")
        out.append("HBM traffic counters, KiB per dispatch as rocprofv3 prints them (one counter per run)")
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            out.append("  command: rocprofv3 --pmc %s --output-format csv -d gpurun_out/pmc_%s_%s -o pmc -- python3 bench.py "
                       "--workload %s --steps 2 --warmup 1 --no-cpu-baseline --no-32k --no-mfma-ceiling --traffic-calibration"
                       % (c, "fetch" if c[0] == "F" else "write", wl, wl))
        if "copy_1GiB" in f and "copy_1GiB" in w:
            ff, wf = GIB_KIB / f["copy_1GiB"][1], GIB_KIB / w["copy_1GiB"][1]
            out.append("  scale from the 1 GiB copy (reads 1 GiB, writes 1 GiB): FETCH_SIZE x%.3f, WRITE_SIZE x%.3f" % (ff, wf))
        else:
            ff, wf = 2.0, 1.0
            out.append("  no copy kernel in the runs: scale factors of earlier runs on this pool, FETCH_SIZE x2, WRITE_SIZE x1")
        out.append("  %-28s %14s %14s %16s" % ("kernel", "FETCH_SIZE", "WRITE_SIZE", "bytes (scaled)"))
        for k in f:
            if k in w and not k.startswith("void") and (k.split("<")[0].endswith("_kernel") or k == "copy_1GiB"):
                out.append("  %-28s %14.1f %14.1f %16.0f" % (k, f[k][1], w[k][1], 1024 * (ff * f[k][1] + wf * w[k][1])))
        if args.kernel in f and args.kernel in w:
            out.append("traffic_bytes_per_launch %s %s %.0f" % (wl_name, args.kernel.split("<")[0],
                                                             1024 * (ff * f[args.kernel][1] + wf * w[args.kernel][1])))

    sq = {}
    sq_dirs = sorted(glob.glob(os.path.join(d, "pmc_sq*_" + wl)))
    for sd in sq_dirs:
        cm = counter_means(sd)
        for c, per in (cm or {}).items():
            if args.kernel in per:
                sq[c] = per[args.kernel][1]
    if sq:
        out.append("")
        out.append("SQ counters of %s, mean per launch (one pass of at most eight counters per run)" % args.kernel)
        for sd in sq_dirs:
            out.append("  run: rocprofv3 --pmc <the counters below, eight at a time> --output-format csv -d %s -o pmc -- python3 bench.py "
                       "--workload %s --steps 2 --warmup 1 --no-cpu-baseline --no-32k --no-mfma-ceiling" % (sd, wl))
        for c in sorted(sq):
            out.append("  %-32s %.6g" % (c, sq[c]))
        out.append("  derived:")
        if "SQ_INSTS_MFMA" in sq and "SQ_INSTS_VALU" in sq:
            # SQ_INSTS_VALU counts the MFMAs too
            out.append("    other VALU instructions per MFMA = (SQ_INSTS_VALU - SQ_INSTS_MFMA) / SQ_INSTS_MFMA = %.2f"
                       % (sq["SQ_INSTS_VALU"] / sq["SQ_INSTS_MFMA"] - 1.0))
        if "SQ_VALU_MFMA_BUSY_CYCLES" in sq and "SQ_BUSY_CU_CYCLES" in sq:
            out.append("    matrix pipe busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES) = %.1f%% of the cycles "
                       "the compute units are busy" % (100 * sq["SQ_VALU_MFMA_BUSY_CYCLES"] / (4 * sq["SQ_BUSY_CU_CYCLES"])))
        if "SQ_BUSY_CU_CYCLES" in sq and dur and dur.get(args.kernel):
            ns = sum(dur[args.kernel]) / len(dur[args.kernel])
            out.append("    average shader clock during the launch = SQ_BUSY_CU_CYCLES / 256 CUs / kernel time = %.2f GHz"
                       % (sq["SQ_BUSY_CU_CYCLES"] / 256 / ns))
        if "SQ_LDS_BANK_CONFLICT" in sq and sq.get("SQ_LDS_IDX_ACTIVE"):
            out.append("    LDS bank-conflict cycles / LDS active cycles = %.3f" % (sq["SQ_LDS_BANK_CONFLICT"] / sq["SQ_LDS_IDX_ACTIVE"]))

    text = "\n".join(out) + "\n"
    with open(args.out, "w") as fh:
        fh.write(text)
    sys.stdout.write(text)


if __name__ == "__main__":
    main()
