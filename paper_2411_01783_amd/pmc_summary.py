"""Turn two `rocprofv3 --pmc` runs of `bench.py --pmc-probe` (one collecting FETCH_SIZE, one
WRITE_SIZE) into a short text summary of HBM bytes per kernel launch.

The raw counters are scaled by what the same counters read for the probe's plain streaming
kernel, which reads and writes a known number of bytes; the factor is printed in the
summary.

usage: python -m paper_2411_01783_amd.pmc_summary FETCH.csv WRITE.csv OUT_DIR WORKLOAD "CMD"
"""
from __future__ import annotations

import collections
import csv
import os
import sys

# kernel-name substring -> tag of the summary file (first match wins)
KERNELS = [("prefill_ring_walk_kernel", "prefill_ring_walk_kernel"),
           ("prefill_mfma_kernel", "prefill_mfma_kernel"), ("decode_kernel", "decode_kernel"),
           ("merge_split_kernel", "merge_kernel_split"), ("merge_kernel", "merge_kernel_ring")]
COPY_MARK = "MulFunctor"


def per_dispatch(path: str, counter: str):
    """kernel tag -> list of per-dispatch counter values."""
    acc = collections.defaultdict(lambda: collections.defaultdict(float))
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        name = r["Kernel_Name"]
        tag = None
        if COPY_MARK in name:
            tag = "copy"
        else:
            for k, t in KERNELS:
                if k in name:
                    tag = t
                    break
        if tag is not None:
            acc[tag][r["Dispatch_Id"]] += float(r["Counter_Value"])
    return {k: list(v.values()) for k, v in acc.items()}


def main():
    fetch_csv, write_csv, out_dir, workload, cmd = sys.argv[1:6]
    copy_bytes = 1 << 28
    rd = per_dispatch(fetch_csv, "FETCH_SIZE")
    wr = per_dispatch(write_csv, "WRITE_SIZE")
    rd_copy = sum(rd["copy"]) / len(rd["copy"])
    wr_copy = sum(wr["copy"]) / len(wr["copy"])
    f_rd = copy_bytes / rd_copy   # bytes per counter unit
    f_wr = copy_bytes / wr_copy
    for tag in sorted(set(rd) | set(wr)):
        if tag == "copy":
            continue
        r = rd.get(tag, [0.0])
        w = wr.get(tag, [0.0])
        rb = sum(r) / len(r) * f_rd
        wb = sum(w) / len(w) * f_wr
        wl = workload if tag.startswith("prefill") or tag.endswith("_ring") else "decode_b32"
        path = os.path.join(out_dir, "%s_%s_hbm_traffic.txt" % (tag, wl))
        with open(path, "w") as f:
            f.write("commands (two runs, one counter each):\n  %s\n\n" % cmd)
            f.write("kernel: %s   workload: %s   dispatches: %d\n" % (tag, wl, len(r)))
            f.write("scale reference: elementwise kernel reading and writing %d bytes:\n"
                    "  FETCH_SIZE reads %.1f per dispatch -> %.2f bytes per unit\n"
                    "  WRITE_SIZE reads %.1f per dispatch -> %.2f bytes per unit\n"
                    % (copy_bytes, rd_copy, f_rd, wr_copy, f_wr))
            f.write("FETCH_SIZE per dispatch (mean): %.1f -> %.0f bytes read\n"
                    % (sum(r) / len(r), rb))
            f.write("WRITE_SIZE per dispatch (mean): %.1f -> %.0f bytes written\n"
                    % (sum(w) / len(w), wb))
            f.write("traffic_bytes_per_launch = %.0f\n" % (rb + wb))
        print(path, "%.3e" % (rb + wb))


if __name__ == "__main__":
    main()
