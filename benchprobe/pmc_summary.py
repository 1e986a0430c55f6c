#!/usr/bin/env python3
"""Condenses rocprofv3 CSV output into the short text summaries kept under profiles/.

Input: one or more output directories of `rocprofv3 --kernel-trace --stats --output-format csv` and of
`rocprofv3 --pmc <counters> --output-format csv` runs of ONE command (each counter set needs a run of its own).
Output (stdout, or --out FILE): per kernel whose name contains one of --kernel's substrings the number of dispatches and
the average / minimum / maximum duration from the trace, and the mean of every counter per dispatch.  With --traffic-out
it also writes the file bench.py reads `roofline.traffic` from: the kernel's FETCH_SIZE and WRITE_SIZE readings (KiB per
dispatch), each scaled by what the same counter reads for the benchmark's plain copy kernel of known size (1 GiB read,
1 GiB written), plus the hash of the kernel's sources so that a summary taken before a kernel change is not printed
after it.

    python3 benchprobe/pmc_summary.py --kernel k_decode_split --dirs out/prof/trace out/prof/fetch \\
        out/prof/write --traffic-kernel "k_decode_split<2, false>" --traffic-out profiles/..._traffic.txt
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ATTN_SOURCES = ("paper_2604_04722_amd/csrc/kvq_attn.hip", "paper_2604_04722_amd/csrc/kvq_internal.h",
                "paper_2604_04722_amd/csrc/kvq_quant.h")
COPY_BYTES = 1 << 30          # bench.py's calibration copy: 1 GiB read + 1 GiB written


def sources_sha256(paths=ATTN_SOURCES) -> str:
    h = hashlib.sha256()
    for p in paths:
        with open(os.path.join(ROOT, p), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def short(name: str) -> str:
    name = name.replace("void ", "").replace("kvq::", "").replace("benchprobe::", "")
    cut = name.find("(")
    return name if cut < 0 else name[:cut]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dirs", nargs="+", required=True)
    ap.add_argument("--kernel", nargs="*", default=[], help="substrings of the kernel names to report (default: all)")
    ap.add_argument("--out", default=None)
    ap.add_argument("--traffic-kernel", default=None, help="kernel (short name, exact) whose scaled HBM bytes go to --traffic-out")
    ap.add_argument("--traffic-out", default=None)
    args = ap.parse_args()

    dur = {}                                                    # kernel -> (calls, avg, min, max) from kernel_stats
    ctr = collections.defaultdict(lambda: collections.defaultdict(list))
    for d in args.dirs:
        for f in glob.glob(os.path.join(d, "**", "*_kernel_stats.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                dur[short(r["Name"])] = (int(r["Calls"]), float(r["AverageNs"]), float(r["MinNs"]), float(r["MaxNs"]))
        for f in glob.glob(os.path.join(d, "**", "*_counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                ctr[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))

    def wanted(k):
        return not args.kernel or any(s in k for s in args.kernel)

    lines = []
    if dur:
        lines.append("kernel trace (--kernel-trace --stats): dispatches, average / min / max duration in us")
        for k, (n, avg, mn, mx) in sorted(dur.items(), key=lambda kv: -kv[1][0] * kv[1][1]):
            if wanted(k):
                lines.append("  %-44s n=%-6d avg %10.2f  min %10.2f  max %10.2f" % (k, n, avg / 1e3, mn / 1e3, mx / 1e3))
    if ctr:
        lines.append("counters (--pmc): mean per dispatch (min .. max), n = dispatches")
        for k in sorted(ctr):
            if not wanted(k):
                continue
            for c in sorted(ctr[k]):
                v = ctr[k][c]
                lines.append("  %-44s %-28s %16.1f  (%.1f .. %.1f)  n=%d" % (k, c, sum(v) / len(v), min(v), max(v), len(v)))
    text = "\n".join(lines) + "\n"
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text)

    if args.traffic_out:
        k = args.traffic_kernel
        if k not in ctr or "FETCH_SIZE" not in ctr[k] or "WRITE_SIZE" not in ctr[k]:
            sys.exit("no FETCH_SIZE / WRITE_SIZE readings for kernel %r (have: %s)" % (k, ", ".join(sorted(ctr))))
        cp = ctr.get("k_probe_copy", {})
        if "FETCH_SIZE" not in cp or "WRITE_SIZE" not in cp:
            sys.exit("no FETCH_SIZE / WRITE_SIZE readings for the calibration copy k_probe_copy")
        mean = lambda v: sum(v) / len(v)                         # noqa: E731
        f_fac = COPY_BYTES / 1024.0 / mean(cp["FETCH_SIZE"])
        w_fac = COPY_BYTES / 1024.0 / mean(cp["WRITE_SIZE"])
        rd = mean(ctr[k]["FETCH_SIZE"]) * f_fac * 1024.0
        wr = mean(ctr[k]["WRITE_SIZE"]) * w_fac * 1024.0
        with open(args.traffic_out, "w") as f:
            f.write("# HBM bytes per dispatch of %s from rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE runs (KiB per dispatch),\n"
                    "# each scaled by what the same counter reads for the plain copy of 1 GiB (k_probe_copy): fetch reading x %.4f,\n"
                    "# write reading x %.4f.  bench.py prints this number as roofline.traffic while the kernel's sources still hash\n"
                    "# to the value below.\n" % (k, f_fac, w_fac))
            f.write("kernel=%s\nfetch_KiB=%.1f\nwrite_KiB=%.1f\nfetch_factor=%.4f\nwrite_factor=%.4f\ndispatches=%d\n"
                    % (k, mean(ctr[k]["FETCH_SIZE"]), mean(ctr[k]["WRITE_SIZE"]), f_fac, w_fac, len(ctr[k]["FETCH_SIZE"])))
            f.write("traffic_bytes_per_launch=%.0f\n" % (rd + wr))
            f.write("sources_sha256=%s\n" % sources_sha256())


if __name__ == "__main__":
    main()
