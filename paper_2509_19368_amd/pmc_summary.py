"""Per-kernel averages of a rocprofv3 --pmc counter collection.

Usage: python -m paper_2509_19368_amd.pmc_summary <..._counter_collection.csv> [counter]
Prints, per kernel name, the number of dispatches and the mean / min / max of the counter.
"""
from __future__ import annotations

import csv
import sys
from collections import defaultdict


def summarize(path: str, counter: str | None = None):
    rows = defaultdict(list)
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            if counter and r.get("Counter_Name") != counter:
                continue
            name = r.get("Kernel_Name", "?")
            rows[(name, r.get("Counter_Name", "?"))].append(float(r.get("Counter_Value", "nan")))
    out = []
    for (name, cn), v in sorted(rows.items(), key=lambda kv: -sum(kv[1])):
        out.append((name, cn, len(v), sum(v) / len(v), min(v), max(v)))
    return out


def main():
    if len(sys.argv) < 2:
        print(__doc__)
        sys.exit(2)
    for name, cn, n, mean, lo, hi in summarize(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else None):
        short = name.split("(")[0][-70:]
        print(f"{cn:12s} n={n:6d} mean={mean:14.1f} min={lo:14.1f} max={hi:14.1f}  {short}")


if __name__ == "__main__":
    main()
