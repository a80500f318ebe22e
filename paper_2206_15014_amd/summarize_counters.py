#!/usr/bin/env python3
"""Condense the counter CSVs written by profile_counters.sh into a short text report.

Part 1: per pass directory entry (workload), kernel and grid size, the mean of each counter over the
dispatches after warm-up.  Part 2: figures derived from them per nm_* kernel:
  HBM bytes per launch  = FETCH_SIZE * fetch_factor + WRITE_SIZE * write_factor (KiB), the factors being
                          known bytes / counter reading of the plain 256 MiB copy in the same report
                          (the read counter prices a 128-byte request as 64 bytes on this part);
  MFMA utilisation      = (SQ_VALU_MFMA_BUSY_CYCLES / SIMDs) / (SQ_BUSY_CYCLES / shader engines);
  L2 hit rate           = TCC_HIT / TCC_REQ;  LDS conflict share = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE.
Usage: summarize_counters.py <dir with *_counter_collection.csv> [--simds 1024] [--engines 32]
"""
import collections
import csv
import glob
import os
import re
import sys

COPY_BYTES = 256 << 20


def short(name):
    name = re.sub(r"void nm::\(anonymous namespace\)::|\(nm::GemmArgs.*|\(float const\*.*|void at::native::", "", name)
    return name[:64]


def main():
    d = sys.argv[1]
    simds = int(sys.argv[sys.argv.index("--simds") + 1]) if "--simds" in sys.argv else 1024
    engines = int(sys.argv[sys.argv.index("--engines") + 1]) if "--engines" in sys.argv else 32
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in sorted(glob.glob(os.path.join(d, "*_counter_collection.csv"))):
        tag = os.path.basename(f).replace("_counter_collection.csv", "").split(".")[0]
        for r in csv.DictReader(open(f)):
            key = (tag, short(r["Kernel_Name"]), int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1))
            agg[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
    mean = {}
    print("== counters: mean over the dispatches after the first quarter ==")
    for key, counters in sorted(agg.items()):
        tag, name, grid = key
        if "rocclr" in name and tag != "copy":
            continue                                    # the harness's own small host-to-device copies
        print("%s | %s | workgroups=%d" % key)
        for cname, v in sorted(counters.items()):
            v = v[len(v) // 4:]
            mean[key + (cname,)] = sum(v) / len(v)
            print("    %-32s dispatches=%4d mean=%16.1f" % (cname, len(v), mean[key + (cname,)]))

    def get(key, cname):
        return mean.get(key + (cname,))

    copy_key = next((k for k in agg if k[0] == "copy" and "copyBuffer" in k[1]), None)
    ff = wf = None
    print("\n== derived ==")
    if copy_key is not None and get(copy_key, "FETCH_SIZE") and get(copy_key, "WRITE_SIZE"):
        ff = COPY_BYTES / 1024.0 / get(copy_key, "FETCH_SIZE")
        wf = COPY_BYTES / 1024.0 / get(copy_key, "WRITE_SIZE")
        print("calibration on the 256 MiB copy: FETCH_SIZE factor %.3f, WRITE_SIZE factor %.3f" % (ff, wf))
    for key in sorted(agg):
        tag, name, grid = key
        if not (name.startswith("gemm_") or name.startswith("compress_")):
            continue
        parts = []
        f, w = get(key, "FETCH_SIZE"), get(key, "WRITE_SIZE")
        if f is not None and w is not None and ff is not None:
            parts.append("HBM read %.0f KiB + write %.0f KiB = %.2f MB per launch" % (
                f * ff, w * wf, (f * ff + w * wf) * 1024 / 1e6))
        mb, sb = get(key, "SQ_VALU_MFMA_BUSY_CYCLES"), get(key, "SQ_BUSY_CYCLES")
        if mb and sb:
            parts.append("MFMA utilisation %.1f %%" % (100.0 * (mb / simds) / (sb / engines)))
        h, q = get(key, "TCC_HIT_sum"), get(key, "TCC_REQ_sum")
        if h is not None and q:
            parts.append("L2 hit rate %.0f %%" % (100.0 * h / q))
        c, a = get(key, "SQ_LDS_BANK_CONFLICT"), get(key, "SQ_LDS_IDX_ACTIVE")
        if c is not None and a:
            parts.append("LDS conflict share %.0f %%" % (100.0 * c / a))
        print("%s | %s | workgroups=%d: %s" % (tag, name, grid, "; ".join(parts)))


if __name__ == "__main__":
    main()
