"""Turn two `rocprofv3 --pmc` runs of `bench.py --pmc-probe` (one collecting FETCH_SIZE, one
WRITE_SIZE) into a short text summary of HBM bytes per kernel launch.

The raw counters are scaled by what the same counters read for the probe's plain streaming
kernel, which reads and writes a known number of bytes; the factor is printed in the
summary.

usage: python -m bench_support.pmc_summary FETCH.csv WRITE.csv OUT_DIR WORKLOAD "CMD"

A third run of the same probe with matrix-pipe and LDS counters is summarised by
       python -m bench_support.pmc_summary --mfma COUNTERS.csv OUT_DIR WORKLOAD "CMD"
into <kernel>_<workload>_mfma_counters.txt: mean counter values per launch, the share of
SIMD cycles with the matrix pipe busy, the clock the launch ran at and the FLOPs it executed.

The per-kernel table (one row per kernel and grid) of a `rocprofv3 --kernel-trace --stats
--output-format csv` run of bench.py, together with the JSON line bench.py printed in that very run, is written by
       python -m bench_support.pmc_summary --stats KERNEL_TRACE.csv BENCH_LINE.json OUT.txt "CMD"
"""
from __future__ import annotations

import collections
import csv
import os
import sys

# kernel-name substring -> tag of the summary file (first match wins)
KERNELS = [("prefill_ring_walk_kernel", "prefill_ring_walk_kernel"),
           ("prefill_mfma_kernel", "prefill_mfma_kernel"),
           ("decode_flat_merge_kernel", "decode_flat_merge_kernel"),
           ("decode_flat_kernel", "decode_flat_kernel"), ("decode_kernel", "decode_kernel"),
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


def short_name(name: str) -> str:
    """A readable kernel name: our namespace spelled plainly, argument lists cut. (The
    profiler leaves names with a __bf16 template argument mangled; those are spelled out here.)"""
    import re
    m = re.match(r"_ZN2cp12_GLOBAL__N_1(\d+)", name)
    if m:
        n = int(m.group(1))
        base = name[m.end():m.end() + n]
        rest = name[m.end() + n:]
        args = []
        if rest.startswith("I"):
            i = 1
            while i < len(rest) and rest[i] != "E":
                if rest.startswith("DF16b", i):
                    args.append("__bf16"); i += 5
                elif rest[i] == "f":
                    args.append("float"); i += 1
                elif rest.startswith("Lb", i):
                    args.append("true" if rest[i + 2] == "1" else "false"); i += 4
                elif rest.startswith("Li", i):
                    j = rest.index("E", i)
                    args.append(rest[i + 2:j]); i = j + 1
                else:
                    break
        return "cp::%s%s" % (base, "<%s>" % ", ".join(args) if args else "")
    name = name.replace("(anonymous namespace)::", "")
    if name.startswith("void "):
        name = name[5:]
    cut = name.find("(")
    return name if cut < 0 else name[:cut]


def stats_main():
    """Per (kernel, grid) durations from the kernel trace: the same kernel serves several
    workloads of one bench run (the 128K and the 1M ring walk, ...), told apart by their grids."""
    import json
    trace_csv, bench_json, out, cmd = sys.argv[2:6]
    line = json.loads(open(bench_json).read().strip().splitlines()[-1])
    groups = collections.defaultdict(list)
    in_order = collections.defaultdict(list)   # (start, duration) per group, for the timed region
    for r in csv.DictReader(open(trace_csv)):
        name = short_name(r["Kernel_Name"])
        wg = [int(r["Workgroup_Size_" + a]) for a in "XYZ"]
        grid = tuple(int(r["Grid_Size_" + a]) // w for a, w in zip("XYZ", wg))
        dur = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
        groups[(name, grid)].append(dur)
        in_order[(name, grid)].append((int(r["Start_Timestamp"]), dur))
    total = sum(sum(v) for v in groups.values())
    with open(out, "w") as f:
        f.write("command:\n  %s\n\n" % cmd)
        f.write("bench.py's own line of this run (HIP events around whole driver calls):\n")
        f.write("  value %.2f %s   ms_per_step %.4f   steps %d   warmup %d\n"
                % (line["value"], line["unit"], line["ms_per_step"], line["steps"], line["warmup"]))

        def block(label, b):
            if isinstance(b, dict) and "us_per_launch" in b:
                f.write("  %-58s us_per_launch %10.2f  frac %.4f  %s\n"
                        % (label, b["us_per_launch"], b.get("frac", float("nan")),
                           b.get("kernel", "")[:60]))
        block("roofline", line.get("roofline"))
        for k, v in line.get("aux", {}).items():
            if isinstance(v, dict):
                block("aux.%s.roofline" % k, v.get("roofline"))
            elif isinstance(v, list):
                for e in v:
                    if isinstance(e, dict):
                        tag = e.get("workload", k)
                        block("aux.%s[%s].roofline" % (k, tag), e.get("roofline"))
                        block("aux.%s[%s].roofline_literal_step" % (k, tag),
                              e.get("roofline_literal_step"))
        # The headline's timed region: bench.py's first calls of the ring walk are the warm-up
        # steps, then the timed steps, one launch per virtual rank each.
        n_ranks = line.get("config", {}).get("virtual_ranks", 0)
        head = [(k, v) for k, v in in_order.items() if "prefill_ring_walk_kernel" in k[0]]
        if n_ranks and head:
            key, seq = max(head, key=lambda kv: len(kv[1]))
            seq.sort()
            lo, hi = line["warmup"] * n_ranks, (line["warmup"] + line["steps"]) * n_ranks
            timed = [d for _, d in seq[lo:hi]]
            if len(timed) == hi - lo:
                avg = sum(timed) / len(timed)
                f.write("\ntimed region of the headline (launches %d..%d of %s in dispatch order): "
                        "avg %.1f us, min %.1f, max %.1f; %d x avg = %.3f ms of ms_per_step %.3f\n"
                        % (lo + 1, hi, key[0], avg / 1e3, min(timed) / 1e3, max(timed) / 1e3,
                           n_ranks, n_ranks * avg / 1e6, line["ms_per_step"]))
        f.write("\nper-kernel durations of the same process (rocprofv3 kernel trace), one row per "
                "kernel and grid (workgroups x, y, z):\n")
        f.write("%-64s %-16s %7s %14s %11s %11s %7s %11s %11s\n"
                % ("kernel", "grid", "calls", "total_ns", "avg_ns", "median_ns", "pct", "min_ns",
                   "max_ns"))
        for (name, grid), d in sorted(groups.items(), key=lambda kv: -sum(kv[1])):
            ours = "cp::" in name or "probe_kernel" in name
            if not ours and sum(d) < 5e-4 * total:
                continue
            d.sort()
            f.write("%-64s %-16s %7d %14d %11.0f %11d %7.3f %11d %11d\n"
                    % (name[:64], "%dx%dx%d" % grid, len(d), sum(d), sum(d) / len(d),
                       d[len(d) // 2], 100.0 * sum(d) / total, d[0], d[-1]))
    print(out)


def main():
    if len(sys.argv) > 1 and sys.argv[1] == "--mfma":
        return mfma_main()
    if len(sys.argv) > 1 and sys.argv[1] == "--stats":
        return stats_main()
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
