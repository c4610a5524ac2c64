#!/usr/bin/env python3
"""Benchmark of the per-rank hot path of context-parallel ring attention on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input: for the
default workload (Llama3-405B per-GPU head shape, 128K full prefill, pass-KV) that is the
complete ring of Algorithm 2 over all 16 virtual CP ranks: every rank's queries against the
16 load-balanced KV shards in ring order, merged with Equation 4. The headline runs a rank's
16 ring steps inside one launch (running softmax state in registers, every shard behind an
arrival flag); `aux` also times a launch per ring step with the merge in the attention
epilogues, and with 16 stored partials and a separate merge kernel per rank. Inputs are
resident in HBM before the timed region.

Prints ONE JSON line. `value` is causal-effective TFLOP/s (4 * d * N_H * visible pairs).
`roofline` describes the dominant kernel (the bf16 MFMA attention kernel walking a rank's
ring), timed with HIP events around whole driver calls in a second pass (median of the
timed steps; mean, minimum and maximum beside it). `cpu_baseline` times the fp64 oracle on a
bounded sample of the same workload. `aux` carries the other configurations, each with a
`roofline` block of its own: the literal launch-per-step ring, the merge kernel, the 1M-token
prefill (a subset of ranks), pass-Q decode and the pass-Q partial prefills.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2411_01783_amd import binding as B  # noqa: E402
from paper_2411_01783_amd import workloads as W  # noqa: E402
from bench_support import probes as P  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E


def _i32(x):
    return torch.as_tensor(np.asarray(x, dtype=np.int32)).to("cuda")


def visible_pairs(q_pos: np.ndarray, kv_pos: np.ndarray) -> int:
    """Exact count of (query, key) pairs with kv_pos <= q_pos."""
    ks = np.sort(kv_pos.astype(np.int64))
    return int(np.searchsorted(ks, q_pos.astype(np.int64), side="right").sum())


def event_times(fn, reps: int, warmup: int = 1):
    """HIP-event time of every one of `reps` calls of fn (ms each), on torch's current stream,
    which is the stream the binding launches on."""
    for _ in range(warmup):
        fn()
    out = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1))
    return out


def spread(ms_list, per: float = 1.0):
    """median / mean / min / max of event times, in microseconds per `per` launches."""
    a = np.asarray(ms_list, dtype=np.float64) * 1e3 / per
    return {"us_median": round(float(np.median(a)), 2), "us_mean": round(float(a.mean()), 2),
            "us_min": round(float(a.min()), 2), "us_max": round(float(a.max()), 2),
            "samples": int(a.size)}


def roofline_block(bound: str, kernel: str, work: float, us: float, traffic=None, **extra):
    """`work` = algorithmic FLOPs (mfma) or bytes (hbm) of one launch, `us` = its duration."""
    if bound == "mfma":
        achieved, peak, unit, key = work / us / 1e6, PEAK_BF16_TFLOPS, "TFLOP/s", "flop_per_launch"
    else:
        achieved, peak, unit, key = work / us / 1e3, PEAK_HBM_GBS, "GB/s", "bytes_per_launch"
    blk = {"bound": bound, "kernel": kernel, "achieved": round(achieved, 2), "peak": peak,
           "unit": unit, "frac": round(achieved / peak, 4), "traffic": traffic,
           "us_per_launch": round(us, 2), key: work}
    if traffic is not None:
        blk["traffic_source"] = "profiles/ (rocprofv3 --pmc summary stored in the repository; " \
                                "counters are not read in this run)"
    blk.update(extra)
    return blk


# ---------------------------------------------------------------------------
# pass-KV prefill (the headline workload)
# ---------------------------------------------------------------------------

def build_prefill(w: W.Workload):
    q, k, v = W.qkv(w, device="cuda")
    n = w.n_ranks
    pos = [B.cp_shard_positions(w.t_new, n, r) for r in range(n)]
    idx = [torch.as_tensor(p.astype(np.int64)).to("cuda") for p in pos]
    qs = [q[i].contiguous() for i in idx]
    ks = [k[i].contiguous() for i in idx]
    vs = [v[i].contiguous() for i in idx]
    del q
    ps = [_i32(p) for p in pos]
    # Headline: every rank's N ring steps walked inside ONE launch (running softmax state in
    # registers, so Equation 4 is applied inside the online softmax; shards visited in ring
    # order, each behind its arrival flag - all set here, the shards being resident).
    flags = [torch.ones(n, dtype=torch.int32, device="cuda") for _ in range(n)]
    ring = B.Ring(qs, ks, vs, ps, ps, out_dtype=torch.bfloat16, fused_merge=2, arrived=flags)
    # one launch per ring step, the merge in the attention epilogues (one running fp32 (O, LSE)
    # per rank). One stream: with the drivers' optional second stream consecutive launches
    # overlap, which gains under 1 % here and makes per-kernel durations in a trace meaningless.
    steps = B.Ring(qs, ks, vs, ps, ps, out_dtype=torch.bfloat16, fused_merge=True)
    # scratch for the per-call measurements: 16 fp32 partials and their separate merge
    parts = B.Ring(qs, ks, vs, ps, ps, out_dtype=torch.bfloat16, part_dtype=torch.float32)
    return dict(ring=ring, steps=steps, parts=parts, pos=pos, qs=qs, ks=ks, vs=vs, ps=ps, k_full=k, v_full=v)


def time_steps(fn, steps: int, warmup: int) -> float:
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def kernel_pass_prefill(w: W.Workload, st: dict, ranks):
    """HIP-event time of the partial-attention launches of the given ranks' ring loops.

    One event pair brackets the n back-to-back launches of a rank's loop (events between
    the launches would add a dispatch gap to every one of them), a second pair the merge."""
    n = w.n_ranks
    ring = st["parts"]
    total_ms, total_flop, n_launch = 0.0, 0.0, 0
    merge_list, merge_bytes, merge_all = [], 0.0, 0.0
    ws = ring.workspace
    for kq in ranks:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for j in range(n):
            s = (kq - j) % n
            B.cp_attn_partial(st["qs"][kq], st["ks"][s], st["vs"][s], st["ps"][kq], st["ps"][s],
                              out=ring.partial_out[s], lse=ring.partial_lse[s], workspace=ws)
        e1.record()
        m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        m0.record()
        B.cp_attn_merge([ring.partial_out[s] for s in range(n)],
                        [ring.partial_lse[s] for s in range(n)], out=ring.out[kq],
                        lse_out=ring.lse[kq])
        m1.record()
        torch.cuda.synchronize()
        total_ms += e0.elapsed_time(e1)
        for s in range(n):
            total_flop += 4.0 * w.head_dim * w.n_q_heads * visible_pairs(st["pos"][kq],
                                                                         st["pos"][s])
        n_launch += n
        merge_list.append(m0.elapsed_time(m1))
        # Bytes the merge has to move: every LSE, the O row of every NON-EMPTY partial (a
        # partial whose LSE is -inf has weight zero and its O is never read: a quarter of the
        # (row, step) pairs of the load-balanced ring), and the merged output.
        rows = ring.out[kq].shape[0] * w.n_q_heads
        finite = int(torch.isfinite(ring.partial_lse[:n, :ring.out[kq].shape[0]]).sum().item())
        merge_bytes += finite * w.head_dim * 4 + n * rows * 4 + rows * (w.head_dim * 2 + 4)
        merge_all += n * rows * (w.head_dim * 4 + 4) + rows * (w.head_dim * 2 + 4)
    return dict(ms_per_launch=total_ms / n_launch, flop_per_launch=total_flop / n_launch,
                n_launch=n_launch, merge_ms=float(np.median(merge_list)),
                merge_ms_all=merge_list, merge_bytes=merge_bytes / len(ranks),
                merge_bytes_if_all_read=merge_all / len(ranks))


def per_call_prefill(w: W.Workload, st: dict, reps: int = 8):
    """One cp_attn_partial call at its real shape: an off-diagonal ring step (half of the
    query rows see the whole shard, the others nothing) and the diagonal step."""
    ring = st["parts"]
    out = {}
    kq = w.n_ranks // 2
    for label, s in (("off_diagonal", (kq + 5) % w.n_ranks), ("diagonal", kq)):
        def call():
            B.cp_attn_partial(st["qs"][kq], st["ks"][s], st["vs"][s], st["ps"][kq], st["ps"][s],
                              out=ring.partial_out[s], lse=ring.partial_lse[s],
                              workspace=ring.workspace)
        call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        flop = 4.0 * w.head_dim * w.n_q_heads * visible_pairs(st["pos"][kq], st["pos"][s])
        out[label] = {"us": round(us, 1), "tflops": round(flop / us / 1e6, 1)}
    return out


def cpu_baseline_prefill(w: W.Workload, st: dict, n_tokens: int = 1024):
    """fp64 oracle on a seeded sample of query tokens of the same sequence (all heads)."""
    import oracle
    rng = np.random.default_rng(w.seed)
    tok = np.sort(rng.choice(w.t_new, size=n_tokens, replace=False))
    k64 = W.to_f64(st["k_full"])
    v64 = W.to_f64(st["v_full"])
    # the sampled query rows: regenerate the same seeded q on the device, copy the rows
    q_full, _, _ = W.qkv(w, device="cuda", n_kv=1)
    q64 = W.to_f64(q_full[torch.as_tensor(tok).to("cuda")])
    del q_full
    t0 = time.perf_counter()
    _, _, pairs = oracle.attn(q64, k64, v64, tok, np.arange(w.t_new), return_pairs=True)
    dt = time.perf_counter() - t0
    flop = 4.0 * w.head_dim * w.n_q_heads * pairs
    return dict(value=flop / dt / 1e12, unit="TFLOP/s", cores=oracle.num_threads(), kind="oracle",
                sample="%d seeded query tokens x %d heads vs all visible keys of the %d-token "
                       "sequence (%.2e pairs, %.1f s)" % (n_tokens, w.n_q_heads, w.t_new,
                                                          pairs, dt))


# ---------------------------------------------------------------------------
# split-KV decode (aux; HBM-bound)
# ---------------------------------------------------------------------------

def build_decode(w: W.Workload):
    lengths = W.decode_lengths(w)
    n = w.n_ranks
    ranks = []
    for r in range(n):
        pos, cu = [], [0]
        for b, L in enumerate(lengths):
            p = B.cp_shard_positions(int(L) - 1, n, r)
            if b % n == r:  # round-robin owner of the new token (decode iteration 0)
                p = np.concatenate([p, np.array([L - 1], dtype=np.int32)])
            pos.append(p)
            cu.append(cu[-1] + len(p))
        total = cu[-1]
        ranks.append(dict(
            k=W.normal(w.seed * 100 + 2 * r, (total, w.n_kv_heads, w.head_dim), w.dtype, "cuda"),
            v=W.normal(w.seed * 100 + 2 * r + 1, (total, w.n_kv_heads, w.head_dim), w.dtype,
                       "cuda"),
            kv_pos=_i32(np.concatenate(pos)), cu=_i32(cu), total=total))
    q = W.normal(w.seed * 100 + 99, (w.batch, w.n_q_heads, w.head_dim), w.dtype, "cuda")
    q_pos = _i32(lengths - 1)
    bid = _i32(np.arange(w.batch))
    return dict(ranks=ranks, q=q, q_pos=q_pos, bid=bid, lengths=lengths)


def bench_decode(w: W.Workload, reps: int = 20, graph: bool = True, probe_only: bool = False,
                 cpu: bool = False):
    """Pass-Q decode (Algorithm 4) for 32 sequences x 1 token over 16 virtual ranks, queries
    gathered: every KV holder answers all 32 queries with one launch over its packed KV (the
    ranks' KV are distinct buffers, 1.4 GB in all, so nothing is reused from the 256 MB
    memory-side cache), and one launch merges over splits and holders (Equation 4). Bytes are
    the algorithmic minimum: every K and V element once, Q, O and LSE; the split partials the
    kernels exchange are overhead and not counted."""
    st = build_decode(w)
    n = w.n_ranks
    kv_bytes = sum(2 * r["total"] * w.n_kv_heads * w.head_dim * 2 for r in st["ranks"])
    q_bytes = st["q"].numel() * 2
    out_bytes = w.batch * w.n_q_heads * (w.head_dim * 4 + 4)
    ring_bytes = kv_bytes + n * q_bytes + out_bytes      # every holder reads the gathered Q
    order = np.argsort(np.arange(w.batch) % n, kind="stable")   # rank r owns b with b % n == r
    per = w.batch // n
    q_g, qpos_g, bid_g = st["q"][order].contiguous(), st["q_pos"][order].contiguous(), _i32(order)
    sl = [slice(r * per, (r + 1) * per) for r in range(n)]

    def make_ring(unique):
        return B.Ring([q_g[x] for x in sl], [r["k"] for r in st["ranks"]],
                      [r["v"] for r in st["ranks"]], [qpos_g[x] for x in sl],
                      [r["kv_pos"] for r in st["ranks"]], out_dtype=torch.float32,
                      keep_partials=True, gathered_q=True,
                      cu_seqlens_kv=[r["cu"] for r in st["ranks"]], bid=[bid_g[x] for x in sl],
                      unique_bid=unique)
    gring = make_ring(True)
    if probe_only:
        B.cp_ring_passq_decode(gring)
        torch.cuda.synchronize()
        return None
    ts = event_times(lambda: B.cp_ring_passq_decode(gring), reps, 3)
    us_rank = float(np.median(ts)) * 1e3 / n
    res = dict(workload=w.name, kv_mb_per_rank=round(kv_bytes / n / 1e6, 4),
               launches="per KV holder one decode_flat_kernel over all 32 queries (sequence ids "
                        "unique: CP_SHAPE_UNIQUE_BID); one decode_flat_merge_kernel over splits "
                        "x holders for the whole ring",
               ms_per_rank=round(us_rank / 1e3, 5), gbs=round(ring_bytes / n / us_rank / 1e3, 1),
               frac_hbm=round(ring_bytes / n / us_rank / 1e3 / PEAK_HBM_GBS, 4),
               per_rank=spread(ts, n))
    t_kernel = stored_traffic("decode_flat_kernel", w.name)
    t_merge = stored_traffic("decode_flat_merge_kernel", w.name)
    res["roofline"] = roofline_block(
        "hbm", "decode_flat_kernel (+ 1/16 of the ring's decode_flat_merge_kernel)",
        ring_bytes / n, us_rank,
        None if t_kernel is None or t_merge is None else t_kernel + t_merge / n)
    k_us = stored_kernel_us("cp::decode_flat_kernel", "512x1x1")
    if k_us is not None:
        res["kernel_alone"] = {
            "kernel": "decode_flat_kernel", "us_per_launch": round(k_us, 2),
            "frac_hbm": round(ring_bytes / n / k_us / 1e3 / PEAK_HBM_GBS, 4),
            "source": "profiles/bench_default_run_kernel_stats.txt (rocprofv3 kernel trace of "
                      "the default run, stored in the repository; not measured in this run)"}
    ref = gring.out_all.clone()
    if graph:
        # the same ring replayed from one HIP graph (the paper runs decode under graphs,
        # Section 4.3); the library records kernels only, no memset nodes
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            B.cp_ring_passq_decode(gring)
            side.synchronize()
            g.capture_begin(capture_error_mode="relaxed")
            B.cp_ring_passq_decode(gring)
            g.capture_end()
        torch.cuda.synchronize()
        tg = event_times(g.replay, reps, 3)
        us_g = float(np.median(tg)) * 1e3 / n
        res["graph"] = {"ms_per_rank": round(us_g / 1e3, 5),
                        "gbs": round(ring_bytes / n / us_g / 1e3, 1),
                        "frac_hbm": round(ring_bytes / n / us_g / 1e3 / PEAK_HBM_GBS, 4),
                        "matches_eager": bool(torch.equal(ref, gring.out_all))}
        del g
    # context: the same ring without the promise of unique sequence ids (the split-per-query
    # kernel, a merge launch per holder and a merge across holders), and single calls
    oring = make_ring(False)
    to = event_times(lambda: B.cp_ring_passq_decode(oring), reps, 3)
    res["ring_without_unique_bid"] = {
        "ms_per_rank": round(float(np.median(to)) / n, 5),
        "frac_hbm": round(ring_bytes / n / (float(np.median(to)) * 1e3 / n) / 1e3 / PEAK_HBM_GBS, 4),
        "max_abs_diff": round(float((oring.out_all - ref).abs().max()), 6)}
    del oring
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    lse = torch.empty((w.batch, w.n_q_heads), dtype=torch.float32, device="cuda")
    call_bytes = kv_bytes / n + q_bytes + out_bytes
    for label, uniq in (("single_call_unique_bid", True), ("single_call", False)):
        shape = B.make_shape(B.CP_BF16, w.head_dim, w.n_q_heads, w.n_kv_heads, w.batch,
                             max(r["total"] for r in st["ranks"]), w.batch,
                             flags=B.CP_SHAPE_UNIQUE_BID if uniq else 0)
        ws = torch.empty(B.cp_workspace_bytes(shape, B.CP_WS_DECODE) + 256, dtype=torch.uint8,
                         device="cuda")

        def one_pass():
            for r in st["ranks"]:
                B.cp_attn_decode(st["q"], r["k"], r["v"], st["q_pos"], r["kv_pos"], r["cu"],
                                 st["bid"], out=out, lse=lse, workspace=ws, unique_bid=uniq)
        tc = event_times(one_pass, max(5, reps // 2), 2)
        us_c = float(np.median(tc)) * 1e3 / n
        res[label] = {"us_per_call": round(us_c, 2),
                      "frac_hbm": round(call_bytes / us_c / 1e3 / PEAK_HBM_GBS, 4),
                      "launches": "decode kernel + its own merge over the splits"}
    if cpu:
        # the oracle on one holder's call (all 32 queries against rank 0's packed KV), in full
        import oracle
        r0 = st["ranks"][0]
        q64, k64, v64 = W.to_f64(st["q"]), W.to_f64(r0["k"]), W.to_f64(r0["v"])
        qp = st["q_pos"].cpu().numpy()
        kp = r0["kv_pos"].cpu().numpy()
        cu = r0["cu"].cpu().numpy()
        t0 = time.perf_counter()
        oracle.attn(q64, k64, v64, qp, kp, cu_q=np.arange(w.batch + 1, dtype=np.int32), cu_kv=cu)
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = dict(
            value=round(call_bytes / dt / 1e9, 4), unit="GB/s", cores=oracle.num_threads(),
            kind="oracle", sample="one KV holder's whole call (32 queries x 16 heads against "
                                  "its %d packed keys), %.2f s" % (r0["total"], dt))
    return res


# ---------------------------------------------------------------------------
# KV-cache append (aux; HBM-bound copy): one rank's share of a 128K prefill, then the
# one-token appends of a decode step
# ---------------------------------------------------------------------------

def bench_kv_append(reps: int = 20):
    """`reps` appends recorded in one HIP graph and replayed (issued call by call from Python
    they would be bound by the interpreter, not by the GPU)."""
    def graph_time(fn):
        for _ in range(3):
            fn()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            side.synchronize()
            g.capture_begin(capture_error_mode="relaxed")
            for _ in range(reps):
                fn()
            g.capture_end()
        torch.cuda.synchronize()
        return time_steps(g.replay, 2, 1) / reps     # 3 replays + 3 eager calls in all

    w = W.WORKLOADS["prefill_128k"]
    rows = w.t_new // w.n_ranks                      # 8192 tokens of one sequence per rank
    k_new = W.normal(71, (rows, w.n_kv_heads, w.head_dim), w.dtype, "cuda")
    v_new = W.normal(72, (rows, w.n_kv_heads, w.head_dim), w.dtype, "cuda")
    pos = _i32(B.cp_shard_positions(w.t_new, w.n_ranks, 0))
    cu_new = _i32([0, rows])
    cache = B.KVCache([rows * (3 * reps + 4)], w.n_kv_heads, w.head_dim)
    sec = graph_time(lambda: B.cp_kv_append(cache, k_new, v_new, pos, cu_new))
    moved = 2 * (2 * k_new.numel() * 2) + 2 * rows * 4          # K, V read + written; positions
    res = {"prefill_rows": rows, "prefill_us": sec * 1e6, "prefill_gbs": moved / sec / 1e9,
           "dropped": int(cache.dropped.item())}
    # decode step: the owner of 2 of 32 sequences appends one token each
    d = W.WORKLOADS["decode_b32"]
    cache = B.KVCache([3 * reps + 4] * d.batch, d.n_kv_heads, d.head_dim)
    counts = np.zeros(d.batch, dtype=np.int64)
    counts[[0, d.n_ranks]] = 1
    cu_new = _i32(np.concatenate([[0], np.cumsum(counts)]))
    k2, v2, p2 = k_new[:2].contiguous(), v_new[:2].contiguous(), pos[:2].contiguous()
    sec = graph_time(lambda: B.cp_kv_append(cache, k2, v2, p2, cu_new))
    res["decode_step_us"] = sec * 1e6
    res["dropped"] += int(cache.dropped.item())
    return {k: (round(v, 3) if isinstance(v, float) else v) for k, v in res.items()}


# ---------------------------------------------------------------------------
# persistent-KV partial prefill, pass-Q (aux; launch-bound at small T)
# ---------------------------------------------------------------------------

def bench_partial_prefill(names, reps: int = 5, cpu: bool = False):
    rows = []
    for name in names:
        w = W.WORKLOADS[name]
        q, k, v = W.qkv(w, device="cuda")
        n, p_cached, t_new = w.n_ranks, w.p_cached, w.t_new
        qpos, kvpos = [], []
        for r in range(n):
            qp = B.cp_shard_positions(t_new, n, r, offset=p_cached)
            qpos.append(qp)
            kvpos.append(np.concatenate([B.cp_shard_positions(p_cached, n, r), qp]))

        def take(t, pos):
            return t[torch.as_tensor(pos.astype(np.int64)).to("cuda")].contiguous()
        ring = B.Ring([take(q, pp - p_cached) for pp in qpos], [take(k, pp) for pp in kvpos],
                      [take(v, pp) for pp in kvpos], [_i32(pp) for pp in qpos],
                      [_i32(pp) for pp in kvpos], out_dtype=torch.bfloat16)
        flop = 4.0 * w.head_dim * w.n_q_heads * (t_new * p_cached + t_new * (t_new + 1) // 2)
        row = {"workload": name, "t_new": t_new, "p_cached": p_cached}
        for label, fn in (("passq", B.cp_ring_passq), ("passkv", B.cp_ring_passkv)):
            sec = time_steps(lambda: fn(ring), reps, 2)
            row[label + "_ms_per_ring"] = round(sec * 1e3, 3)
            row[label + "_us_per_call"] = round(sec * 1e6 / (n * n), 2)
            row[label + "_tflops"] = round(flop / sec / 1e12, 1)
        # pass-Q with the (small) query shards gathered: one call per KV holder answers all
        # 16 steps, then the same 16 merges
        m = len(qpos[0])
        q_all = take(q, np.concatenate(qpos) - p_cached)
        qpos_all = _i32(np.concatenate(qpos))
        gring = B.Ring([q_all[r * m:(r + 1) * m] for r in range(n)], ring.tensors[1],
                       ring.tensors[2], [qpos_all[r * m:(r + 1) * m] for r in range(n)],
                       ring.tensors[4], out_dtype=torch.bfloat16, keep_partials=True,
                       gathered_q=True)
        sec = time_steps(lambda: B.cp_ring_passq(gring), reps, 2)
        row["passq_gathered_ms_per_ring"] = round(sec * 1e3, 3)
        row["passq_gathered_us_per_rank"] = round(sec * 1e6 / n, 2)
        row["passq_gathered_tflops"] = round(flop / sec / 1e12, 1)
        # Roofline of the gathered call of one KV holder (+ 1/16 of the one merge launch).
        # The arithmetic intensity is (T/N) * 16 FLOP per KV byte: memory-bound at T = 128
        # (every holder reads its 4.2 MB of K and V once), matrix-bound from T = 1024 on.
        kv_bytes_rank = sum(int(t.numel()) * 2 * 2 for t in ring.tensors[1]) / n
        io_bytes_rank = t_new * w.n_q_heads * w.head_dim * 2 + \
            (t_new // n) * w.n_q_heads * (w.head_dim * 2 + 4)
        kern = "prefill_mfma_kernel (KV axis split over grid.z) + merge_split_kernel"
        if t_new * 16 / n < 315:
            row["roofline"] = roofline_block("hbm", kern, kv_bytes_rank + io_bytes_rank,
                                             sec * 1e6 / n)
        else:
            row["roofline"] = roofline_block("mfma", kern, flop / n, sec * 1e6 / n)
        row["roofline_literal_step"] = roofline_block(
            "mfma", kern + ", one launch per ring step (Algorithm 3 as printed)",
            flop / (n * n), row["passq_us_per_call"])
        row["passq_gathered_max_abs_diff"] = round(max(
            float((a.float() - b.float()).abs().max()) for a, b in zip(gring.out, ring.out)), 5)
        if cpu and t_new <= 128:
            # the oracle's own pass-Q ring (Algorithm 3: 16 x 16 partial attentions + 16 merges)
            import oracle
            q64 = [W.to_f64(x) for x in ring.tensors[0]]
            k64 = [W.to_f64(x) for x in ring.tensors[1]]
            v64 = [W.to_f64(x) for x in ring.tensors[2]]
            t0 = time.perf_counter()
            oracle.ring_passq(q64, k64, v64, qpos, kvpos)
            dt = time.perf_counter() - t0
            row["cpu_baseline"] = dict(value=round(flop / dt / 1e12, 5), unit="TFLOP/s",
                                       cores=oracle.num_threads(), kind="oracle",
                                       sample="the whole pass-Q ring of this workload, %.2f s" % dt)
        del gring
        rows.append(row)
        del ring, q, k, v
        torch.cuda.empty_cache()
    return rows


def selector_table(c_flops: float):
    """Orders cp_select_order picks for the partial-prefill workloads, with C = the
    attention rate measured above and BW = one xGMI link (153 GB/s) or a 50 GB/s NIC."""
    out = []
    for bw_name, bw in (("xgmi_153GBs", 153e9), ("nic_50GBs", 50e9)):
        for t in (128, 1024, 2048, 8192, 16384, 131072):
            p = 131072 if t < 131072 else 0
            order = B.cp_select_order(t, p, 128, 8, 16, c_flops, bw, 2.0, B.CP_RULE_ANALYTIC)
            out.append({"link": bw_name, "t_new": t, "p_cached": p,
                        "order": "pass-KV" if order == B.CP_ORDER_PASS_KV else "pass-Q"})
    return out


# ---------------------------------------------------------------------------
# HBM traffic (hardware counters)
# ---------------------------------------------------------------------------

PROBE_COPY_BYTES = 1 << 28


def mfma_rate_probe(iters: int = 20000, reps: int = 3):
    """What a bare loop of bf16 MFMAs sustains on this part, for zero and for N(0,1) operands
    (the second draws more power and settles at a lower clock): context for roofline.frac."""
    n_wg = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(n_wg * 512, dtype=torch.float32, device="cuda")
    n_el = P.OPERAND_BYTES // 2
    out = {}
    for name, ops in (("zeros", torch.zeros(n_el, dtype=torch.bfloat16, device="cuda")),
                      ("normal", W.normal(77, (n_el,), "bf16", "cuda"))):
        best = 0.0
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flop = P.mfma_rate(ops, iters, n_wg, sink)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, flop / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        out["tflops_%s_operands" % name] = round(best, 1)
    out["workgroups"] = n_wg
    return out


def bench_paper_step_shapes(reps: int = 10):
    """One ring step at the two shapes whose attention time the paper prints (its breakdown
    table for P + T = 128000 on CP4: T = 3200 and T = 12800, i.e. 800 / 3200 query tokens x 16
    heads against a 32000-token KV shard): context next to the H100 figures, not a target."""
    rows = []
    n = 4
    for t_new, paper_us in ((3200, 414.0), (12800, 1608.0)):
        p_cached = 128000 - t_new
        qp = [B.cp_shard_positions(t_new, n, r, offset=p_cached) for r in range(n)]
        kvp = [np.concatenate([B.cp_shard_positions(p_cached, n, r), qp[r]]) for r in range(n)]
        q = W.normal(81, (len(qp[0]), 16, 128), "bf16", "cuda")
        k = W.normal(82, (len(kvp[1]), 1, 128), "bf16", "cuda")
        v = W.normal(83, (len(kvp[1]), 1, 128), "bf16", "cuda")
        q_pos, kv_pos = _i32(qp[0]), _i32(kvp[1])
        shape = B.make_shape(B.CP_BF16, 128, 16, 1, q.shape[0], k.shape[0])
        ws = torch.empty(B.cp_workspace_bytes(shape, B.CP_WS_PARTIAL) + 256, dtype=torch.uint8,
                         device="cuda")
        out = torch.empty((q.shape[0], 16, 128), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((q.shape[0], 16), dtype=torch.float32, device="cuda")

        def call():
            B.cp_attn_partial(q, k, v, q_pos, kv_pos, out=out, lse=lse, workspace=ws)
        call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        flop = 4.0 * 128 * 16 * visible_pairs(qp[0], kvp[1])
        rows.append({"t_new": t_new, "q_tokens": int(q.shape[0]), "kv_tokens": int(k.shape[0]),
                     "us": round(us, 1), "tflops": round(flop / us / 1e6, 1),
                     "paper_h100_us": paper_us})
    return rows


def hbm_read_probe(nbytes: int, n_buffers: int = 16, reps: int = 5):
    """What one launch that only reads `nbytes` once achieves (ramp and tail included), cycling
    over `n_buffers` buffers as the decode measurement cycles over the ranks' KV (no reuse from
    the 256 MB memory-side cache): the yardstick for the decode kernel."""
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    bufs = [torch.ones(nbytes // 4, dtype=torch.float32, device="cuda") for _ in range(n_buffers)]
    out = {"bytes": nbytes, "us_by_wg_per_cu": {}}
    best = None
    for wg_per_cu in (1, 2, 3, 4):
        n_wg = n_cu * wg_per_cu
        sink = torch.empty(n_wg * 256, dtype=torch.int32, device="cuda")

        def one_pass():
            for b in bufs:
                P.hbm_read(b, n_wg, sink)
        sec = time_steps(one_pass, reps, 2) / n_buffers
        out["us_by_wg_per_cu"][str(wg_per_cu)] = round(sec * 1e6, 2)
        best = sec if best is None else min(best, sec)
    out["best_us"] = round(best * 1e6, 2)
    out["best_gbs"] = round(nbytes / best / 1e9, 1)
    out["best_frac_hbm"] = round(nbytes / best / 1e9 / PEAK_HBM_GBS, 4)
    return out


def pmc_probe(st):
    """The work the counter runs profile: a streaming kernel that reads and writes
    PROBE_COPY_BYTES (the scale reference), one pass-KV ring pass in one launch per rank, one
    with a launch per step and stored partials (and their merge), one decode pass."""
    src = torch.ones(PROBE_COPY_BYTES // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.mul(src, 2.0, out=dst)
    torch.cuda.synchronize()
    B.cp_ring_passkv(st["ring"])
    torch.cuda.synchronize()
    B.cp_ring_passkv(st["parts"])
    torch.cuda.synchronize()
    bench_decode(W.WORKLOADS["decode_b32"], probe_only=True)
    print("pmc probe done")


def stored_kernel_us(kernel: str, grid: str):
    """Average duration (us) of a kernel and grid in the committed kernel-trace summary of the
    default bench run, or None."""
    path = os.path.join(ROOT, "profiles", "bench_default_run_kernel_stats.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 5 and f[0] == kernel and f[1] == grid:
            return float(f[4]) / 1e3
    return None


def stored_traffic(kernel: str, workload: str):
    """Bytes of HBM traffic per launch from the committed counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "%s_%s_hbm_traffic.txt" % (kernel, workload))
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            return float(line.split("=")[1])
    return None


def bench_prefill_1m_subset(ranks=(0, 9), reps: int = 3):
    """The 1M-token pass-KV prefill (the largest configuration) on a subset of the 16 virtual
    ranks: every rank sees the same number of visible pairs by construction, so two ranks'
    ring walks (64K query tokens each against all sixteen 64K-token KV shards) stand for the
    ring. Only the chosen ranks' queries are generated; all KV shards are."""
    w = W.WORKLOADS["prefill_1m"]
    n = w.n_ranks
    _, k, v = W.qkv(w, device="cuda", n_q=1)
    pos = [B.cp_shard_positions(w.t_new, n, r) for r in range(n)]
    idx = [torch.as_tensor(p.astype(np.int64)).to("cuda") for p in pos]
    ks = [k[i].contiguous() for i in idx]
    vs = [v[i].contiguous() for i in idx]
    del k, v
    ps = [_i32(p) for p in pos]
    empty_q = torch.empty((0, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
    empty_p = torch.empty((0,), dtype=torch.int32, device="cuda")
    qs = [W.normal(w.seed * 3 + 100 + r, (len(pos[r]), w.n_q_heads, w.head_dim), w.dtype, "cuda")
          if r in ranks else empty_q for r in range(n)]
    qps = [ps[r] if r in ranks else empty_p for r in range(n)]
    flags = [torch.ones(n, dtype=torch.int32, device="cuda") for _ in range(n)]
    ring = B.Ring(qs, ks, vs, qps, ps, out_dtype=torch.bfloat16, fused_merge=2, arrived=flags)
    ts = event_times(lambda: B.cp_ring_passkv(ring), reps, 1)
    pairs = sum(visible_pairs(pos[r], np.arange(w.t_new)) for r in ranks)
    flop_rank = 4.0 * w.head_dim * w.n_q_heads * pairs / len(ranks)
    us = float(np.median(ts)) * 1e3 / len(ranks)
    res = {"workload": w.name, "ranks_timed": list(ranks), "of_ranks": n,
           "tokens": w.t_new, "ms_per_rank": round(us / 1e3, 3),
           "tflops": round(flop_rank / us / 1e6, 2), "per_rank": spread(ts, len(ranks)),
           "roofline": roofline_block("mfma", "prefill_ring_walk_kernel", flop_rank, us)}
    del ring, qs, ks, vs
    torch.cuda.empty_cache()
    return res


def bench_padded_shards(w: W.Workload, st: dict, reps: int):
    """The headline ring with one padded query token (CP_POS_PAD_Q) in every rank's shard,
    as Algorithm 2 pads shards to equal length: time against the unpadded ring."""
    n = w.n_ranks
    qps = []
    for r in range(n):
        pp = st["ps"][r].clone()
        pp[5::1024] = B.CP_POS_PAD_Q      # 8 padded tokens per shard, in 8 different wavefronts
        qps.append(pp)
    ring = B.Ring(st["qs"], st["ks"], st["vs"], qps, st["ps"], out_dtype=torch.bfloat16,
                  fused_merge=2)
    ts = event_times(lambda: B.cp_ring_passkv(ring), reps, 2)
    return float(np.median(ts))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="prefill_128k",
                    choices=["prefill_128k", "prefill_1m"])
    ap.add_argument("--no-aux", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="also time the headline's launches on all-zero Q, K, V (the kernel's "
                         "efficiency in cycles: the part holds its full clock on such data); off "
                         "by default so that a kernel trace of the default run holds the ring "
                         "walk on N(0,1) data only")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="run one ring pass, one decode pass and a plain streaming kernel of "
                         "known size, then exit (the workload of the rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the ring is simulated over virtual CP ranks on a "
              "single MI355X and no multi-GPU path exists in this build (got --gpus %d)"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.load()
    P.load()

    w = W.WORKLOADS[args.workload]
    st = build_prefill(w)
    ring = st["ring"]
    if args.pmc_probe:
        pmc_probe(st)
        return
    sec = time_steps(lambda: B.cp_ring_passkv(ring), args.steps, args.warmup)
    t = w.t_new
    flop_step = 4.0 * w.head_dim * w.n_q_heads * (t * (t + 1) // 2)
    tflops = flop_step / sec / 1e12

    # dominant kernel: the ring walk, one launch per rank; HIP events around a whole driver call
    # (16 launches and one tile-bound pre-pass over all shards), once per timed step
    walk_ms = event_times(lambda: B.cp_ring_passkv(ring), args.steps, 0)
    us_per_launch = float(np.median(walk_ms)) * 1e3 / w.n_ranks
    flop_per_launch = flop_step / w.n_ranks     # every rank sees the same number of pairs
    kp = kernel_pass_prefill(w, st, ranks=list(range(w.n_ranks)))
    result = {
        "metric": "per-rank partial-attn+merge TFLOP/s (% bf16 MFMA peak); decode HBM GB/s",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "order": "pass-KV", "virtual_ranks": w.n_ranks,
                   "tokens": t, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim,
                   "launches": "one per rank: its 16 ring steps are walked inside the kernel, "
                               "each shard behind an arrival flag (all set: shards resident)",
                   "merge": "Equation 4 inside the online softmax (running state in registers)",
                   "flops": "causal-effective 4*d*N_H*pairs",
                   "ms_per_rank": round(sec * 1e3 / w.n_ranks, 3)},
        "frac_of_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline_block(
            "mfma", "prefill_ring_walk_kernel", flop_per_launch, us_per_launch,
            stored_traffic("prefill_ring_walk_kernel", w.name),
            launches=w.n_ranks * args.steps, per_launch=spread(walk_ms, w.n_ranks),
            timing="median over the timed steps of a HIP-event pair around one driver call "
                   "(16 launches), divided by 16"),
        "aux": {},
    }
    aux = result["aux"]
    # The literal Algorithm 2: one cp_attn_partial launch per ring step into a stored fp32
    # partial, then the merge kernel over the rank's 16 partials.
    us_step = kp["ms_per_launch"] * 1e3
    aux["per_step_launch"] = {
        "what": "Algorithm 2 as printed: a launch per ring step (prefill_mfma_kernel), stored "
                "partials, merge kernel",
        "roofline": roofline_block("mfma", "prefill_mfma_kernel", kp["flop_per_launch"], us_step,
                                   stored_traffic("prefill_mfma_kernel", w.name),
                                   launches=kp["n_launch"])}
    aux["merge"] = {
        "what": "merge_kernel over the 16 fp32 partials of one rank (Equation 4); bytes = every "
                "LSE, the O rows of the non-empty partials, the merged output",
        "ms": round(kp["merge_ms"], 4), "per_launch": spread(kp["merge_ms_all"]),
        "bytes_if_every_partial_were_read": kp["merge_bytes_if_all_read"],
        "roofline": roofline_block("hbm", "merge_kernel", kp["merge_bytes"], kp["merge_ms"] * 1e3,
                                   stored_traffic("merge_kernel_ring", w.name))}
    aux["per_call"] = per_call_prefill(w, st)
    if not args.no_aux and w.name == "prefill_128k":
        # a launch per ring step with stored partials and the merge kernel: fp32 partials, and
        # bf16 partials (the width the paper's All2All model assumes)
        parts = st["parts"]
        secp = time_steps(lambda: B.cp_ring_passkv(parts), args.steps, args.warmup)
        aux["ring_separate_merge_fp32_partials"] = {
            "tflops": round(flop_step / secp / 1e12, 2),
            "frac_of_peak": round(flop_step / secp / 1e12 / PEAK_BF16_TFLOPS, 4),
            "ms_per_rank": round(secp * 1e3 / w.n_ranks, 3)}
        ring16 = B.Ring(st["qs"], st["ks"], st["vs"], st["ps"], st["ps"], out_dtype=torch.bfloat16,
                        part_dtype=torch.bfloat16)
        sec16 = time_steps(lambda: B.cp_ring_passkv(ring16), args.steps, args.warmup)
        aux["ring_separate_merge_bf16_partials"] = {
            "tflops": round(flop_step / sec16 / 1e12, 2),
            "frac_of_peak": round(flop_step / sec16 / 1e12 / PEAK_BF16_TFLOPS, 4),
            "ms_per_rank": round(sec16 * 1e3 / w.n_ranks, 3)}
        del ring16
        # one launch per ring step, Equation 4 in the attention epilogues
        stp = st["steps"]
        secs = time_steps(lambda: B.cp_ring_passkv(stp), args.steps, args.warmup)
        aux["ring_launch_per_step_merge_in_epilogues"] = {
            "tflops": round(flop_step / secs / 1e12, 2),
            "frac_of_peak": round(flop_step / secs / 1e12 / PEAK_BF16_TFLOPS, 4),
            "ms_per_rank": round(secs * 1e3 / w.n_ranks, 3),
            "max_abs_diff_vs_headline": round(max(
                float((a.float() - b.float()).abs().max()) for a, b in zip(stp.out, ring.out)), 5)}
        # the headline's walk without arrival flags
        walk = B.Ring(st["qs"], st["ks"], st["vs"], st["ps"], st["ps"], out_dtype=torch.bfloat16,
                      fused_merge=2)
        tw = event_times(lambda: B.cp_ring_passkv(walk), args.steps, 2)
        secw = float(np.median(tw)) * 1e-3
        aux["ring_walk_without_arrival_flags"] = {
            "tflops": round(flop_step / secw / 1e12, 2),
            "ms_per_rank": round(secw * 1e3 / w.n_ranks, 3)}
        del walk
        # the same ring with padded query tokens in every shard (Algorithm 2 pads shards)
        pad_ms = bench_padded_shards(w, st, args.steps)
        aux["ring_walk_with_padded_queries"] = {
            "ms_per_rank": round(pad_ms / w.n_ranks, 3),
            "vs_unpadded_walk": round(pad_ms * 1e-3 / secw, 4)}
        if args.zero_inputs:
            # the headline's launches on all-zero Q, K, V (same positions, same tile walk, same
            # instruction stream): the part then holds its full clock, so this is the kernel's
            # efficiency in cycles; with N(0,1) data the matrix pipe's switching activity lowers
            # the clock (see mfma_rate_probe) and the same cycles take longer
            zeros = B.Ring([torch.zeros_like(x) for x in st["qs"]],
                           [torch.zeros_like(x) for x in st["ks"]],
                           [torch.zeros_like(x) for x in st["vs"]], st["ps"], st["ps"],
                           out_dtype=torch.bfloat16, fused_merge=2)
            secz = time_steps(lambda: B.cp_ring_passkv(zeros), args.steps, args.warmup)
            aux["ring_walk_on_zero_inputs"] = {
                "tflops": round(flop_step / secz / 1e12, 2),
                "frac_of_peak": round(flop_step / secz / 1e12 / PEAK_BF16_TFLOPS, 4)}
            del zeros
        # context: the same per-rank result from ONE launch per rank over the whole sequence's
        # K/V in natural order (what an all-gather of KV instead of a ring would run): no ring
        # steps, so none of their per-launch start-up, epilogue and merge traffic
        kv_pos_all = _i32(np.arange(w.t_new))
        outs = [torch.empty_like(o) for o in ring.out]
        lses = [torch.empty_like(l) for l in ring.lse]
        ws_shape = B.make_shape(B.CP_BF16, w.head_dim, w.n_q_heads, w.n_kv_heads,
                                st["qs"][0].shape[0], w.t_new)
        ws_all = torch.empty(B.cp_workspace_bytes(ws_shape, B.CP_WS_PARTIAL) + 256,
                             dtype=torch.uint8, device="cuda")

        def all_kv():
            for r in range(w.n_ranks):
                B.cp_attn_partial(st["qs"][r], st["k_full"], st["v_full"], st["ps"][r],
                                  kv_pos_all, out=outs[r], lse=lses[r], workspace=ws_all)
        seca = time_steps(all_kv, args.steps, args.warmup)
        aux["one_launch_per_rank_over_all_kv"] = {
            "tflops": round(flop_step / seca / 1e12, 2),
            "ms_per_rank": round(seca * 1e3 / w.n_ranks, 3),
            "max_abs_diff_vs_headline": round(max(
                float((a.float() - b.float()).abs().max()) for a, b in zip(outs, ring.out)), 5)}
        del outs, lses, ws_all
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline_prefill(w, st)
    del st, ring
    torch.cuda.empty_cache()
    if not args.no_aux:
        if w.name == "prefill_128k":
            aux["prefill_1m"] = bench_prefill_1m_subset()
        aux["decode"] = bench_decode(W.WORKLOADS["decode_b32"], reps=max(20, args.steps),
                                     cpu=not args.no_cpu)
        torch.cuda.empty_cache()
        aux["hbm_read_probe"] = hbm_read_probe(
            int(aux["decode"]["kv_mb_per_rank"] * 1e6) // 4096 * 4096)
        torch.cuda.empty_cache()
        aux["partial_prefill"] = bench_partial_prefill(
            ["partial_prefill_128k_t128", "partial_prefill_128k_t1024",
             "partial_prefill_128k_t2048", "partial_prefill_128k_t8192"], cpu=not args.no_cpu)
        aux["paper_step_shapes"] = bench_paper_step_shapes()
        aux["kv_append"] = bench_kv_append()
        aux["selector"] = selector_table(tflops * 1e12)
        aux["mfma_rate_probe"] = mfma_rate_probe()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
