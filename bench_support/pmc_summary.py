"""Turn two `rocprofv3 --pmc` runs of `bench.py --pmc-probe` (one collecting FETCH_SIZE, one
WRITE_SIZE) into a short text summary of HBM bytes per kernel launch.

The raw counters are scaled by what the same counters read for the probe's plain streaming
kernel, which reads and writes a known number of bytes; the factor is printed in the
summary.

usage: python -m paper_2411_01783_amd.pmc_summary FETCH.csv WRITE.csv OUT_DIR WORKLOAD "CMD"

A third run of the same probe with matrix-pipe and LDS counters is summarised by
       python -m paper_2411_01783_amd.pmc_summary --mfma COUNTERS.csv OUT_DIR WORKLOAD "CMD"
into <kernel>_<workload>_mfma_counters.txt: mean counter values per launch, the share of
SIMD cycles with the matrix pipe busy, the clock the launch ran at and the FLOPs it executed.
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


N_XCD, N_CU, SIMD_PER_CU = 8, 256, 4   # MI355X
FLOP_PER_MOP = 512                      # SQ_INSTS_VALU_MFMA_MOPS_*: 512 operations per count


def mfma_main():
    path, out_dir, workload, cmd = sys.argv[2:6]
    acc = collections.defaultdict(lambda: collections.defaultdict(lambda: collections.defaultdict(float)))
    dur = collections.defaultdict(dict)
    for r in csv.DictReader(open(path)):
        tag = None
        for k, t in KERNELS:
            if k in r["Kernel_Name"]:
                tag = t
                break
        if tag is None:
            continue
        acc[tag][r["Dispatch_Id"]][r["Counter_Name"]] += float(r["Counter_Value"])
        dur[tag][r["Dispatch_Id"]] = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    for tag, disp in sorted(acc.items()):
        if not tag.startswith("prefill"):
            continue  # launches of a few microseconds: the counters' window is not the kernel's
        n = len(disp)
        mean = collections.defaultdict(float)
        for d in disp.values():
            for c, v in d.items():
                mean[c] += v / n
        ns = sum(dur[tag].values()) / n
        wl = workload if tag.startswith("prefill") or tag.endswith("_ring") else "decode_b32"
        out = os.path.join(out_dir, "%s_%s_mfma_counters.txt" % (tag, wl))
        with open(out, "w") as f:
            f.write("command:\n  %s\n\n" % cmd)
            f.write("kernel: %s   workload: %s   dispatches: %d   mean duration %.1f us\n"
                    % (tag, wl, n, ns / 1e3))
            for c in sorted(mean):
                f.write("  %-32s %.4g per launch\n" % (c, mean[c]))
            cycles = mean.get("GRBM_GUI_ACTIVE", 0.0) / N_XCD   # summed over the XCDs
            if cycles > 0:
                f.write("clock during the launch: %.2f GHz (GRBM_GUI_ACTIVE / %d XCDs / duration)\n"
                        % (cycles / ns, N_XCD))
                busy = mean.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0)
                f.write("matrix pipe busy: %.1f %% of SIMD cycles (SQ_VALU_MFMA_BUSY_CYCLES / "
                        "(cycles x %d CUs x %d SIMDs))\n"
                        % (100.0 * busy / (cycles * N_CU * SIMD_PER_CU), N_CU, SIMD_PER_CU))
            mops = mean.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0.0)
            if mops > 0:
                f.write("bf16 MFMA operations executed: %.4g FLOP per launch (%d per counted MOP), "
                        "%.1f TFLOP/s over the mean duration\n"
                        % (mops * FLOP_PER_MOP, FLOP_PER_MOP, mops * FLOP_PER_MOP / ns / 1e3))
        print(out)


def main():
    if len(sys.argv) > 1 and sys.argv[1] == "--mfma":
        return mfma_main()
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
