"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws random numbers and names workload shapes. It holds none
of the method's arithmetic (no sharding, no masks, no attention): the oracle and
the HIP library each derive positions and shards on their own from the same
full-sequence tensors.

The paper evaluates on synthetic context lengths fed to Llama3-405B with TP8
inside a node, so one GPU sees 16 query heads and 1 KV head of dimension 128
(Section 4.1). Post-RoPE projections are stood in for by i.i.d. N(0,1) draws in
fp32, rounded once to the storage dtype; both sides consume the rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str            # "passkv_prefill" | "passq_prefill" | "passq_decode"
    n_ranks: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str           # "bf16" | "fp32"
    t_new: int = 0       # new tokens T (prefill)
    p_cached: int = 0    # cached tokens P (partial prefill)
    batch: int = 1       # decode batch
    len_lo: int = 0      # decode KV length range (inclusive), counts the new token
    len_hi: int = 0
    seed: int = 0


WORKLOADS = {
    # tiny full ring: 512 tokens, GQA 4:1, d=64, fp32, 2 virtual ranks
    "tiny_passkv": Workload("tiny_passkv", "passkv_prefill", 2, 4, 1, 64, "fp32",
                            t_new=512, seed=1001),
    # Llama3-405B per-GPU shape, 128K full prefill, 16 virtual ranks (8K tokens each)
    "prefill_128k": Workload("prefill_128k", "passkv_prefill", 16, 16, 1, 128, "bf16",
                             t_new=131072, seed=1002),
    # 1M full prefill, 16 virtual ranks (64K tokens each)
    "prefill_1m": Workload("prefill_1m", "passkv_prefill", 16, 16, 1, 128, "bf16",
                           t_new=1048576, seed=1003),
    # persistent-KV partial prefill, pass-Q: 128K cached, T new tokens
    "partial_prefill_128k_t128": Workload("partial_prefill_128k_t128", "passq_prefill", 16, 16,
                                          1, 128, "bf16", t_new=128, p_cached=131072, seed=1004),
    "partial_prefill_128k_t1024": Workload("partial_prefill_128k_t1024", "passq_prefill", 16, 16,
                                           1, 128, "bf16", t_new=1024, p_cached=131072,
                                           seed=1004),
    "partial_prefill_128k_t2048": Workload("partial_prefill_128k_t2048", "passq_prefill", 16, 16,
                                           1, 128, "bf16", t_new=2048, p_cached=131072,
                                           seed=1004),
    "partial_prefill_128k_t8192": Workload("partial_prefill_128k_t8192", "passq_prefill", 16, 16,
                                           1, 128, "bf16", t_new=8192, p_cached=131072,
                                           seed=1004),
    # batched decode: 32 sequences x 1 token, KV lengths uniform in [32K, 128K]
    "decode_b32": Workload("decode_b32", "passq_decode", 16, 16, 1, 128, "bf16",
                           batch=32, len_lo=32768, len_hi=131072, seed=1005),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "fp32": torch.float32}[name]


def normal(seed: int, shape, dtype: str = "bf16", device: str = "cpu",
           chunk_rows: int = 1 << 16) -> torch.Tensor:
    """N(0,1) tensor drawn in fp32 from a seeded generator, rounded to `dtype`.

    Drawn in row chunks so that million-token tensors never hold an fp32 copy.
    The stream depends on (seed, device type), so one run must draw on one device.
    """
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    out = torch.empty(shape, dtype=torch_dtype(dtype), device=device)
    rows = shape[0]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen,
                                 dtype=torch.float32, device=device).to(out.dtype)
    return out


def qkv(w: Workload, device: str = "cpu", n_q: Optional[int] = None,
        n_kv: Optional[int] = None):
    """Full-sequence q [T, N_H, d], k, v [P+T, N_KV, d] for a prefill workload."""
    n_q = w.t_new if n_q is None else n_q
    n_kv = w.p_cached + w.t_new if n_kv is None else n_kv
    q = normal(w.seed * 3 + 0, (n_q, w.n_q_heads, w.head_dim), w.dtype, device)
    k = normal(w.seed * 3 + 1, (n_kv, w.n_kv_heads, w.head_dim), w.dtype, device)
    v = normal(w.seed * 3 + 2, (n_kv, w.n_kv_heads, w.head_dim), w.dtype, device)
    return q, k, v


def decode_lengths(w: Workload) -> np.ndarray:
    """KV length of every sequence in the decode batch, counting the new token."""
    rng = np.random.default_rng(w.seed)
    return rng.integers(w.len_lo, w.len_hi + 1, size=w.batch).astype(np.int64)


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact upcast of a (possibly bf16, possibly device) tensor to a NumPy fp64 array."""
    return t.detach().to("cpu", torch.float64).numpy()
