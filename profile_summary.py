#!/usr/bin/env python3
"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python3 profile_summary.py stats    <dir>/<name>_kernel_stats.csv        OUT.txt --cmd "<command that made it>" [--trace <name>_kernel_trace.csv]
    python3 profile_summary.py traffic  <fetch>_counter_collection.csv <write>_counter_collection.csv OUT.txt \
                                        --workload xlarge --cmd "<the two commands>"
    python3 profile_summary.py counters <pmc>_counter_collection.csv OUT.txt --cmd "<command>" [--durations STATS.txt]

stats:    per-kernel calls / total / average / share from `rocprofv3 --kernel-trace --stats` (libsgnn's kernels only).
traffic:  HBM bytes per launch from two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch), each
          scaled by what the same counter reads for copy_f32_kernel moving 256 MiB (`bench.py --calibrate-copy`).
          Lines "traffic <kernel> <bytes>" are read back by bench.py (roofline.traffic).
counters: per-kernel averages of whatever counters a `--pmc` run collected, and the ratios SQ_VALU_MFMA_BUSY_CYCLES /
          SQ_BUSY_CU_CYCLES (matrix pipe busy share) and SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES where both are present.
Kernel names are shortened the way bench.py names its groups (tile, transposes, operand type for the GEMMs).
"""
from __future__ import annotations

import argparse
import collections
import csv
import re

SKIP = ("at::", "rocprim", "Cijk", "__amd_rocclr", "vectorized", "elementwise_kernel", "hipcub", "radix", "index_")


def short(n: str) -> str:
    n = n.replace("(anonymous namespace)::", "").replace("void ", "")
    n = re.sub(r"\((?:[^()]|\([^()]*\))*\)$", "", n).strip()
    m = re.match(r"gemm_(fast_)?kernel<(\d+), (\d+), \d+, \d+, (\w+), (\w+), (\w+)(, \w+)*>", n)
    if m:
        return "gemm_kernel<%sx%s,%s%s,%s>" % (m.group(2), m.group(3), "T" if m.group(4) == "true" else "N",
                                                 "T" if m.group(5) == "true" else "N", "bf16" if m.group(6) == "true" else "f32")
    m = re.match(r"gemm_direct_kernel<(\d+), \d+, \d+, (\w+), (\w+), (\w+)>", n)
    if m:
        # bench.py files the direct-to-LDS kernel under gemm_kernel with its tile shape
        return "gemm_kernel<%sx128,%s%s,f32>" % (m.group(1), "T" if m.group(2) == "true" else "N",
                                                 "T" if m.group(3) == "true" else "N")
    if n.startswith("gemm_thin_tn_kernel"):
        return "gemm_kernel<thin32,TN,f32>"
    if n.startswith("gemm_smallk_nt_kernel"):
        return "gemm_kernel<smallk,NT,f32>"
    m = re.match(r"(spmm_main_kernel)<(\d+), (\d+), .*?(true|false)>", n)
    if m:      # the last template argument: the instantiation with the loss in its epilogue
        return "%s<%s,%s%s>" % (m.group(1), m.group(2), m.group(3), ",xent" if m.group(4) == "true" else "")
    return re.sub(r"<.*>$", "", n)


def ours(name: str) -> bool:
    return not any(s in name for s in SKIP)


def cmd_stats(args):
    rows = [r for r in csv.DictReader(open(args.inputs[0])) if ours(r["Name"])]
    agg = collections.OrderedDict()
    for r in rows:
        a = agg.setdefault(short(r["Name"]), [0, 0, 10 ** 18, 0])
        a[0] += int(r["Calls"]); a[1] += int(r["TotalDurationNs"]); a[2] = min(a[2], int(r["MinNs"])); a[3] = max(a[3], int(r["MaxNs"]))
    tot = sum(a[1] for a in agg.values())
    lines = ["# rocprofv3 --kernel-trace --stats summary (kernels of libsgnn; torch's input-generation kernels omitted)",
             "# command: " + args.cmd]
    if args.note:
        lines.append("# " + args.note)
    lines.append("%-44s %7s %12s %12s %7s %10s %10s" % ("kernel", "calls", "total_us", "avg_us", "pct", "min_us", "max_us"))
    for k, a in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        lines.append("%-44s %7d %12.1f %12.2f %6.2f%% %10.2f %10.2f" % (k[:44], a[0], a[1] / 1e3, a[1] / a[0] / 1e3,
                                                                         100.0 * a[1] / tot, a[2] / 1e3, a[3] / 1e3))
    if args.trace:
        # dispatches that overlapped no other dispatch in time: what HIP events around a kernel on an otherwise idle chip see
        ev = []
        for r in csv.DictReader(open(args.trace)):
            ev.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]))
        ev.sort()
        alone = collections.OrderedDict()
        max_end_before = 0
        for i, (b, e, name) in enumerate(ev):
            overl = b < max_end_before or (i + 1 < len(ev) and ev[i + 1][0] < e)
            max_end_before = max(max_end_before, e)
            if not ours(name):
                continue
            a = alone.setdefault(short(name), [0, 0, 0, 0])
            a[2] += 1; a[3] += e - b
            if not overl:
                a[0] += 1; a[1] += e - b
        lines.append("")
        lines.append("# dispatches that overlapped no other dispatch in time (from the kernel trace of the same run): the figure that")
        lines.append("# bench.py's event-bracketed single-stream pass measures")
        lines.append("%-44s %7s %12s %14s %14s" % ("kernel", "alone", "avg_us", "overlapped", "avg_us"))
        for k, a in sorted(alone.items(), key=lambda kv: -kv[1][3]):
            no, to = a[0], a[1]
            ov, tov = a[2] - a[0], a[3] - a[1]
            lines.append("%-44s %7d %12s %14d %14s" % (k[:44], no, "%.2f" % (to / no / 1e3) if no else "-", ov,
                                                        "%.2f" % (tov / ov / 1e3) if ov else "-"))
    open(args.out, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines[:16]))


def _load(path, counter=None):
    acc = collections.defaultdict(lambda: collections.defaultdict(lambda: [0, 0.0]))
    for r in csv.DictReader(open(path)):
        if counter and r["Counter_Name"] != counter:
            continue
        if not ours(r["Kernel_Name"]):
            continue
        a = acc[short(r["Kernel_Name"])][r["Counter_Name"]]
        a[0] += 1; a[1] += float(r["Counter_Value"])
    return acc


def cmd_traffic(args):
    F = {k: v["FETCH_SIZE"] for k, v in _load(args.inputs[0], "FETCH_SIZE").items()}
    W = {k: v["WRITE_SIZE"] for k, v in _load(args.inputs[1], "WRITE_SIZE").items()}
    copy_kib = 256 * 1024.0
    fc, wc = F["copy_f32_kernel"], W["copy_f32_kernel"]
    ff, wf = copy_kib / (fc[1] / fc[0]), copy_kib / (wc[1] / wc[0])
    lines = ["# HBM traffic per kernel launch, %s workload, from two rocprofv3 counter runs:" % args.workload,
             "#   " + args.cmd,
             "# Counters are in KiB per dispatch, averaged over the dispatches of a kernel, and scaled by what the same counter",
             "# reads for copy_f32_kernel moving 256 MiB (--calibrate-copy): FETCH_SIZE read %.1f KiB -> factor %.3f;" % (fc[1] / fc[0], ff),
             "# WRITE_SIZE read %.1f KiB -> factor %.3f." % (wc[1] / wc[0], wf),
             "# Kernels are keyed as bench.py names them, averaged over all their shapes in the step.",
             "# columns: kernel  dispatches  FETCH_SIZE_KiB  WRITE_SIZE_KiB  read_bytes  written_bytes",
             "# lines starting with 'traffic' are read by bench.py: kernel, total HBM bytes per launch"]
    keys = sorted((k for k in F if k in W), key=lambda k: -(F[k][1] * ff + W[k][1] * wf))
    tr = []
    for k in keys[:20]:
        fa, wa = F[k][1] / F[k][0], W[k][1] / W[k][0]
        rb, wb = fa * ff * 1024, wa * wf * 1024
        lines.append("%-40s %6d %12.1f %12.1f %14.0f %14.0f" % (k, F[k][0], fa, wa, rb, wb))
        tr.append("traffic %s %.0f" % (k, rb + wb))
    open(args.out, "w").write("\n".join(lines + tr) + "\n")
    print("\n".join(lines + tr))


def cmd_counters(args):
    acc = _load(args.inputs[0])
    names = sorted({c for v in acc.values() for c in v})
    lines = ["# rocprofv3 --pmc counters per kernel launch (averages over the dispatches of a kernel)", "# command: " + args.cmd]
    if args.note:
        lines.append("# " + args.note)
    dur = {}
    if args.durations:       # a "stats" summary of the same workload: average duration per kernel
        for ln in open(args.durations):
            f = ln.split()
            if len(f) >= 7 and f[-5].replace(".", "").isdigit() and not ln.startswith("#"):
                dur[" ".join(f[:-6])] = float(f[-4])
    lines.append("# mfma_busy = SQ_VALU_MFMA_BUSY_CYCLES / SQ_BUSY_CU_CYCLES as collected (the first is summed over the four SIMDs of a")
    lines.append("# compute unit: divide by 4 for a per-SIMD share); mfma_share = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x average")
    lines.append("# duration x 2.4 GHz), the share of the launch during which a SIMD's matrix pipe was busy at the nominal clock")
    lines.append("%-40s %6s " % ("kernel", "disp") + " ".join("%24s" % n[-24:] for n in names) + "   mfma_busy  wait_share  mfma_share")
    for k, v in sorted(acc.items(), key=lambda kv: -sum(x[1] for x in kv[1].values())):
        n = max(x[0] for x in v.values())
        avg = {c: v[c][1] / v[c][0] for c in v}
        busy = avg["SQ_VALU_MFMA_BUSY_CYCLES"] / avg["SQ_BUSY_CU_CYCLES"] if "SQ_VALU_MFMA_BUSY_CYCLES" in avg and avg.get("SQ_BUSY_CU_CYCLES") else None
        wait = avg["SQ_WAIT_INST_ANY"] / avg["SQ_WAVE_CYCLES"] if "SQ_WAIT_INST_ANY" in avg and avg.get("SQ_WAVE_CYCLES") else None
        lines.append("%-40s %6d " % (k[:40], n) + " ".join("%24.1f" % avg.get(c, float("nan")) for c in names) +
                     "   %9s  %10s" % ("%.3f" % busy if busy is not None else "-", "%.3f" % wait if wait is not None else "-") +
                     ("  %10.3f" % (avg["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024.0 * dur[k] * 2400.0))
                      if k in dur and "SQ_VALU_MFMA_BUSY_CYCLES" in avg else "  %10s" % "-"))
    open(args.out, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines[:14]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["stats", "traffic", "counters"])
    ap.add_argument("inputs", nargs="+")
    ap.add_argument("--cmd", default="")
    ap.add_argument("--note", default="")
    ap.add_argument("--workload", default="")
    ap.add_argument("--trace", default="", help="stats: the kernel trace CSV of the same run (adds the table of dispatches that ran alone)")
    ap.add_argument("--durations", default="", help="counters: a stats summary of the same workload (adds mfma_share)")
    args = ap.parse_args()
    args.out = args.inputs.pop()
    {"stats": cmd_stats, "traffic": cmd_traffic, "counters": cmd_counters}[args.what](args)


if __name__ == "__main__":
    main()
