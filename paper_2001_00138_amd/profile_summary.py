#!/usr/bin/env python3
"""Turns rocprofv3 CSV output into the short text summaries kept under ``profiles/``.

    python -m paper_2001_00138_amd.profile_summary stats DIR_OR_CSV --command "..." [--title "..."]
        kernel | calls | total ms | average us | % of GPU time   (from *_kernel_stats.csv)

    python -m paper_2001_00138_amd.profile_summary counters CSV [CSV ...] --command "..."
            [--copy-kernel REGEX --copy-bytes N] [--json OUT.json]
        per kernel and counter: dispatches, mean value (from *_counter_collection.csv).
        FETCH_SIZE / WRITE_SIZE are reported in bytes per dispatch (rocprofv3 gives KiB).  With
        --copy-kernel/--copy-bytes the same counters of a plain copy kernel that moved N bytes
        (N read + N written) give the scale factor applied to every other kernel, and --json
        writes {kernel: {"fetch_bytes": .., "write_bytes": ..}} for ``bench.py --traffic-json``.

Output goes to stdout; redirect it into ``profiles/<kernel>_<workload>.txt``.
"""

from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import re
import sys
from collections import defaultdict


def short_name(kernel: str, limit: int = 110) -> str:
    """Kernel names as rocprofv3 prints them, without torch's template noise."""
    k = re.sub(r"\s+", " ", kernel.strip())
    return k if len(k) <= limit else k[:limit - 3] + "..."


def _find(path: str, suffix: str) -> str:
    if os.path.isdir(path):
        hits = sorted(glob.glob(os.path.join(path, "**", f"*{suffix}"), recursive=True))
        if not hits:
            raise FileNotFoundError(f"no *{suffix} under {path}")
        return hits[0]
    return path


def stats_table(csv_path: str, top: int = 12):
    rows = list(csv.DictReader(open(csv_path, newline="")))
    out = []
    for r in rows[:top]:
        out.append((short_name(r["Name"]), int(r["Calls"]), float(r["TotalDurationNs"]) / 1e6,
                    float(r["AverageNs"]) / 1e3, float(r["Percentage"])))
    return out


def counter_means(csv_paths):
    """{kernel: {counter: (dispatches, mean)}} over every dispatch in the files."""
    acc = defaultdict(lambda: defaultdict(list))
    for p in csv_paths:
        for r in csv.DictReader(open(p, newline="")):
            acc[short_name(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (len(v), sum(v) / len(v)) for c, v in cs.items()} for k, cs in acc.items()}


KIB_COUNTERS = ("FETCH_SIZE", "WRITE_SIZE")


def traffic_bytes(means, copy_kernel=None, copy_bytes=None):
    """Bytes per dispatch of FETCH_SIZE / WRITE_SIZE per kernel, scaled by what the copy
    kernel (which read and wrote `copy_bytes`) shows for the same counter."""
    scale = {c: 1.0 for c in KIB_COUNTERS}
    if copy_kernel and copy_bytes:
        pat = re.compile(copy_kernel)
        for c in KIB_COUNTERS:
            seen = [m[c][1] * 1024.0 for k, m in means.items() if pat.search(k) and c in m]
            if seen:
                scale[c] = copy_bytes / (sum(seen) / len(seen))
    out = {}
    for k, m in means.items():
        row = {}
        if "FETCH_SIZE" in m:
            row["fetch_bytes"] = m["FETCH_SIZE"][1] * 1024.0 * scale["FETCH_SIZE"]
        if "WRITE_SIZE" in m:
            row["write_bytes"] = m["WRITE_SIZE"][1] * 1024.0 * scale["WRITE_SIZE"]
        if row:
            out[k] = row
    return out, scale


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("stats")
    a.add_argument("path")
    a.add_argument("--command", required=True, help="the full command that produced the trace")
    a.add_argument("--title", default="rocprofv3 kernel-trace stats")
    b = sub.add_parser("counters")
    b.add_argument("paths", nargs="+")
    b.add_argument("--command", required=True)
    b.add_argument("--title", default="rocprofv3 counter collection")
    b.add_argument("--only", default="patdnn", help="regex of the kernels to list (copy kernel is always listed)")
    b.add_argument("--copy-kernel", default=None)
    b.add_argument("--copy-bytes", type=float, default=None)
    b.add_argument("--json", default=None)
    args = ap.parse_args(argv)

    if args.what == "stats":
        path = _find(args.path, "kernel_stats.csv")
        print(f"# {args.title}")
        print(f"# command (run from /tmp with TMPDIR=/tmp):\n#   {args.command}")
        print("# columns: kernel | calls | total ms | average us | % of GPU time\n")
        for name, calls, total_ms, avg_us, pct in stats_table(path):
            print(f"{name} | {calls} | {total_ms:.2f} | {avg_us:.1f} | {pct:.2f}")
        return 0

    paths = [_find(p, "counter_collection.csv") for p in args.paths]
    means = counter_means(paths)
    traffic, scale = traffic_bytes(means, args.copy_kernel, args.copy_bytes)
    only = re.compile(args.only)
    copy = re.compile(args.copy_kernel) if args.copy_kernel else None
    print(f"# {args.title}")
    print(f"# command (run from /tmp with TMPDIR=/tmp):\n#   {args.command}")
    if copy:
        print(f"# copy kernel /{args.copy_kernel}/ moved {args.copy_bytes:.0f} B each way; "
              f"scale FETCH_SIZE x{scale['FETCH_SIZE']:.4f}, WRITE_SIZE x{scale['WRITE_SIZE']:.4f}")
    print("# columns: counter | dispatches | mean per dispatch\n")
    for k in sorted(means):
        if not (only.search(k) or (copy and copy.search(k))):
            continue
        print(k)
        for c, (n, mean) in sorted(means[k].items()):
            print(f"    {c} | {n} | {mean:.6g}")
        for key, val in traffic.get(k, {}).items():
            print(f"    {key} (scaled) | {val:.6g}")
    if args.json:
        with open(args.json, "w") as f:
            json.dump({k: v for k, v in traffic.items() if only.search(k) and not (copy and copy.search(k))},
                      f, indent=1, sort_keys=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
