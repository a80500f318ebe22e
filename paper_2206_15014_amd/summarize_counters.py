#!/usr/bin/env python3
"""Condense the counter CSVs written by profile_counters.sh into a short text table:
per kernel (and grid size), the mean of each counter over the dispatches after warm-up."""
import collections
import csv
import glob
import os
import re
import sys


def main():
    d = sys.argv[1]
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in sorted(glob.glob(os.path.join(d, "*_counter_collection.csv"))):
        tag = os.path.basename(f).replace("_counter_collection.csv", "").split(".")[0]
        for r in csv.DictReader(open(f)):
            name = re.sub(r"void nm::\(anonymous namespace\)::|\(nm::GemmArgs.*|\(float const\*.*|void at::native::", "", r["Kernel_Name"])[:64]
            key = (tag, name, int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1))
            agg[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
    for (tag, name, grid), counters in sorted(agg.items()):
        print("%s | %s | workgroups=%d" % (tag, name, grid))
        for cname, v in sorted(counters.items()):
            v = v[len(v) // 4:]
            print("    %-32s dispatches=%4d mean=%16.1f" % (cname, len(v), sum(v) / len(v)))


if __name__ == "__main__":
    main()
