"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2411_09688_amd.rocprof_summary stats <dir>          # --kernel-trace --stats run
    python -m paper_2411_09688_amd.rocprof_summary pmc <dir> <COUNTER>  # --pmc run: mean counter per dispatch

Reads only the CSV files rocprofv3 wrote; prints plain text.
"""
from __future__ import annotations

import csv
import glob
import os
import sys
from collections import defaultdict


def _find(d, suffix):
    hits = sorted(glob.glob(os.path.join(d, "**", f"*{suffix}"), recursive=True))
    if not hits:
        raise SystemExit(f"no *{suffix} under {d}")
    return hits[0]


def stats(d):
    rows = [r for r in csv.DictReader(open(_find(d, "kernel_stats.csv"))) if "rocclr" not in r["Name"]]
    # percentages over the kernels listed (the runtime's own copy kernels are left out)
    total = sum(float(r["AverageNs"]) * int(r["Calls"]) for r in rows) or 1.0
    print(f"{'kernel':72s} {'calls':>7s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}")
    for r in rows:
        share = 100.0 * float(r["AverageNs"]) * int(r["Calls"]) / total
        print(f"{r['Name'][:72]:72s} {r['Calls']:>7s} {float(r['AverageNs']) / 1e3:9.2f} {float(r['MinNs']) / 1e3:9.2f} "
              f"{float(r['MaxNs']) / 1e3:9.2f} {share:6.2f}")


def pmc(d, counter):
    path = _find(d, "counter_collection.csv")
    acc = defaultdict(lambda: [0.0, 0])
    for r in csv.DictReader(open(path)):
        if r.get("Counter_Name") != counter:
            continue
        a = acc[r["Kernel_Name"]]
        a[0] += float(r["Counter_Value"])
        a[1] += 1
    print(f"{'kernel':72s} {'dispatches':>10s} {'mean ' + counter:>18s}")
    for k, (tot, n) in sorted(acc.items(), key=lambda kv: -kv[1][0]):
        print(f"{k[:72]:72s} {n:10d} {tot / n:18.2f}")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 4 and sys.argv[1] == "pmc":
        pmc(sys.argv[2], sys.argv[3])
    else:
        raise SystemExit(__doc__)
