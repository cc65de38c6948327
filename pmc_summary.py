#!/usr/bin/env python3
"""Averages rocprofv3 --pmc counter output per kernel.

    python pmc_summary.py DIR [DIR ...] [--kernel SUBSTRING]

Every DIR is the -d directory of one `rocprofv3 --pmc ... --output-format csv` run (one pass of
counters).  Prints, for every kernel whose name contains SUBSTRING (default: all), the number of
dispatches and the mean of every counter over them.  Text only; nothing here touches the GPU.
"""
from __future__ import annotations

import csv
import glob
import os
import sys
from collections import defaultdict


def main():
    args = sys.argv[1:]
    want = ""
    if "--kernel" in args:
        i = args.index("--kernel")
        want = args[i + 1]
        del args[i:i + 2]
    acc = defaultdict(lambda: defaultdict(lambda: [0.0, 0]))   # kernel -> counter -> [sum, n]
    for d in args:
        for path in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            with open(path, newline="") as f:
                for row in csv.DictReader(f):
                    k = row.get("Kernel_Name", "")
                    if want not in k:
                        continue
                    a = acc[k][row["Counter_Name"]]
                    a[0] += float(row["Counter_Value"])
                    a[1] += 1
    for k in sorted(acc):
        print(k)
        for c in sorted(acc[k]):
            s, n = acc[k][c]
            print(f"    {c:36s} dispatches {n:5d}   mean {s / n:16.1f}")


if __name__ == "__main__":
    main()
