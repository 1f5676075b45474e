#!/usr/bin/env python3
"""Turns rocprofv3 CSV output of `bench.py` runs into the short records kept under profiles/.

    python -m paper_2201_05500_amd.profile_summary NAME TRACE_DIR FETCH_DIR WRITE_DIR [--note TEXT]

TRACE_DIR: output of  rocprofv3 --kernel-trace --stats --output-format csv -d TRACE_DIR -- python3 bench.py ...
FETCH_DIR: output of  rocprofv3 --pmc FETCH_SIZE --output-format csv -d FETCH_DIR -- python3 bench.py ...
WRITE_DIR: output of  rocprofv3 --pmc WRITE_SIZE --output-format csv -d WRITE_DIR -- python3 bench.py ...
(the same bench.py arguments in all three).  Writes profiles/NAME_kernels.txt (per-kernel durations and counter
values) and profiles/NAME_step_traffic.json (HBM bytes per launch of every kernel, which bench.py reports as
`roofline.traffic`), stamped with the commit and the hash of the kernel sources they were measured on.

The counters are scaled by what they read for the 1 GiB copies of the library's own copy kernel, which bench.py
runs before its timed region (known traffic: 1 GiB read, 1 GiB written per launch).
"""
import argparse
import collections
import csv
import glob
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KERNEL = "k_stream_copy"
COPY_KIB = float(1 << 20)


def _one(pattern):
    """the newest match: a directory that was profiled into twice holds both runs' files"""
    g = sorted(glob.glob(pattern, recursive=True), key=os.path.getmtime)
    return g[-1] if g else None


def _short(name):
    name = name.split("(")[0].replace("void ", "")
    return name[:70]


def _bare(name):
    """ctr::k_pool<16> -> k_pool"""
    n = _short(name)
    n = n[n.rfind("::") + 2:] if "::" in n else n
    return n.split("<")[0]


def kernel_stats(trace_dir):
    f = _one(trace_dir + "/**/*_kernel_stats.csv")
    rows = []
    if f:
        for r in csv.DictReader(open(f)):
            rows.append((_short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                         float(r["MaxNs"]) / 1e3, r["Percentage"]))
    return rows


def counters(d):
    by = collections.OrderedDict()
    f = _one(d + "/**/*_counter_collection.csv")
    if f:
        for r in csv.DictReader(open(f)):
            by.setdefault(_short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    return by


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("name")
    ap.add_argument("trace_dir")
    ap.add_argument("fetch_dir")
    ap.add_argument("write_dir")
    ap.add_argument("--note", default="")
    ap.add_argument("--command", default="", help="the bench.py command line that was profiled")
    ap.add_argument("--out-dir", default=os.path.join(ROOT, "profiles"), help="where the two files are written")
    ap.add_argument("--steps", type=int, default=0,
                    help="steps the profiled command ran (warm-up + timed); default: the launches of the push kernel")
    a = ap.parse_args()
    sys.path.insert(0, ROOT)
    from paper_2201_05500_amd.build import source_hash

    stats = kernel_stats(a.trace_dir)
    F, W = counters(a.fetch_dir), counters(a.write_dir)
    ours = lambda n: "ctr::" in n
    lines = []
    lines.append("rocprofv3 summary `%s`%s" % (a.name, (": " + a.note) if a.note else ""))
    if a.command:
        lines.append("commands (from the repository root on the GPU box):")
        lines.append("  rocprofv3 --kernel-trace --stats --output-format csv -d %s -- %s" % (a.trace_dir, a.command))
        lines.append("  rocprofv3 --pmc FETCH_SIZE --output-format csv -d %s -- %s" % (a.fetch_dir, a.command))
        lines.append("  rocprofv3 --pmc WRITE_SIZE --output-format csv -d %s -- %s" % (a.write_dir, a.command))
        lines.append("  python3 -m paper_2201_05500_amd.profile_summary %s %s %s %s%s" % (
            a.name, a.trace_dir, a.fetch_dir, a.write_dir, (" --steps %d" % a.steps) if a.steps else ""))
    lines.append("")
    lines.append("== rocprofv3 --kernel-trace --stats (the library's kernels; GEMM kernels of the tower if any)")
    lines.append("%-72s %6s %10s %10s %10s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "pct"))
    for n, calls, avg, mn, mx, pct in stats:
        if ours(n) or "Cijk" in n:
            lines.append("%-72s %6d %10.1f %10.1f %10.1f %7s" % (n, calls, avg, mn, mx, pct))

    copy_f = [v for k, vs in F.items() if COPY_KERNEL in k for v in vs]
    copy_w = [v for k, vs in W.items() if COPY_KERNEL in k for v in vs]
    if not copy_f or not copy_w:
        raise SystemExit("no %s dispatches in the counter runs: cannot calibrate" % COPY_KERNEL)
    med = lambda v: sorted(v)[len(v) // 2]
    scale_f, scale_w = COPY_KIB / med(copy_f), COPY_KIB / med(copy_w)
    lines.append("")
    lines.append("calibration on %d launches of ctr::%s (1 GiB read + 1 GiB written each): FETCH_SIZE median %.0f KiB, "
                 "WRITE_SIZE median %.0f KiB -> scale factors fetch x%.3f, write x%.3f" % (
                     len(copy_f), COPY_KERNEL, med(copy_f), med(copy_w), scale_f, scale_w))
    lines.append("")
    lines.append("== rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE (KiB per dispatch as counted; LAST dispatch of each "
                 "kernel = the steady-most step; GB = scaled)")
    lines.append("%-72s %6s %14s %14s %9s" % ("kernel", "calls", "FETCH_KiB", "WRITE_KiB", "GB"))
    steps = a.steps or max([len(v) for k, v in F.items() if "k_push_span<" in k] or [1])
    rec = {"kernels": {}, "step": {"fetch_KiB": 0.0, "write_KiB": 0.0}}
    for k, vs in F.items():
        if not ours(k) or COPY_KERNEL in k or "k_table_clear" in k:
            continue
        f_last, w_last = vs[-1], (W.get(k) or [0.0])[-1]
        gb = (f_last * scale_f + w_last * scale_w) * 1024 / 1e9
        lines.append("%-72s %6d %14.0f %14.0f %9.2f" % (k, len(vs), f_last, w_last, gb))
        per_step = len(vs) / float(steps)
        bare = _bare(k)
        ent = rec["kernels"].setdefault(bare, {"fetch_KiB": 0.0, "write_KiB": 0.0, "launches_per_step": 0.0})
        if ent["launches_per_step"] == 0.0:       # one entry per kernel family: the figure is per launch
            ent["fetch_KiB"], ent["write_KiB"] = f_last, w_last
        ent["launches_per_step"] += per_step
        rec["step"]["fetch_KiB"] += f_last * per_step
        rec["step"]["write_KiB"] += w_last * per_step
    step_gb = (rec["step"]["fetch_KiB"] * scale_f + rec["step"]["write_KiB"] * scale_w) * 1024 / 1e9
    lines.append("")
    lines.append("whole step (every library kernel, last dispatch x launches per step, scaled): %.2f GB" % step_gb)

    try:
        commit = subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], text=True).strip()
    except Exception:
        commit = None
    rec.update({"workload": a.name, "scale": {"fetch": scale_f, "write": scale_w}, "commit": commit,
                "source_hash": source_hash(), "command": a.command,
                "note": "KiB per launch as counted by rocprofv3 (last dispatch of the run); bytes = KiB * 1024 * scale"})
    lines.append("measured on commit %s, kernel source hash %s" % (commit, rec["source_hash"]))
    out_dir = a.out_dir
    with open(os.path.join(out_dir, "%s_kernels.txt" % a.name), "w") as f:
        f.write("\n".join(lines) + "\n")
    with open(os.path.join(out_dir, "%s_traffic.json" % a.name), "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
