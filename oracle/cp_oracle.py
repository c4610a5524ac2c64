"""fp64 CPU oracle: attention with LSE, merge, load-balanced sharding, ring drivers.

TEST INFRASTRUCTURE ONLY (tests, smoke check, benchmark CPU baseline). Shares
no code with the HIP library and never imports it.

The two numeric kernels (`attn`, `merge`) live in ``cp_oracle.c`` and are the
defining formulas of Appendix B written out. Everything in this file is index
bookkeeping that follows the paper's own steps:

* `shard_positions`        - Section 3.5.1, load-balanced sharding: 2N chunks,
                             rank i takes chunks i and 2N-1-i.
* `ring_passkv`            - Algorithm 2 (ring pass-KV), one KV shard per step,
                             s = (k - j) mod N, merge after the loop.
* `ring_passq`             - Algorithm 3 (ring pass-Q), partial outputs land on
                             the rank that holds the KV and are returned to the
                             query's source rank (the All2All) before merging.
* `ring_passq_decode`      - Algorithm 4 (batched ring pass-Q decode) with the
                             batch ids travelling with the queries.
* `KVCache`                - the persistent per-rank KV cache of multi-turn
                             inference (Sections 3.5.2, 3.6): every turn's new
                             K/V, decode tokens included, are appended to the
                             owning rank's share; `decode_owner` is Section
                             3.6's round-robin placement.
* `select_order`           - pass-KV / pass-Q choice (Section 3.3 Algorithm 1,
                             Appendix C Algorithm 5, Appendix D) from the roofline
                             latencies of Table 1, not from the rearranged tests.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cp_oracle.c")
_LIB = os.path.join(_HERE, "libcp_oracle.so")
_lib = None

INT32_MAX = np.iinfo(np.int32).max


def build(force: bool = False) -> str:
    """Compile cp_oracle.c with gcc (fp64, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_attn.restype = ctypes.c_int64
        lib.oracle_attn.argtypes = [dp, dp, dp, ip, ip, ip, ip, ctypes.c_int32,
                                    ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                    ctypes.c_int32, ctypes.c_int32, ctypes.c_double, dp, dp]
        lib.oracle_merge.restype = None
        lib.oracle_merge.argtypes = [ctypes.POINTER(dp), ctypes.POINTER(dp), ctypes.c_int32,
                                     ctypes.c_int64, ctypes.c_int32, dp, dp]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _iptr(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.POINTER(ctypes.c_int32)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


# --------------------------------------------------------------------------
# Appendix B: attention with log-sum-exp, and Equation 4
# --------------------------------------------------------------------------

def attn(q, k, v, q_pos, kv_pos, cu_q=None, cu_kv=None, scale: Optional[float] = None,
         return_pairs: bool = False):
    """(O, LSE) of q [Tq, N_H, d] against k, v [Tkv, N_KV, d] in fp64.

    Key j is visible to query i iff both belong to the same packed sequence and
    kv_pos[j] <= q_pos[i]. Rows with no visible key give O = 0, LSE = -inf.
    The softmax scale defaults to 1/sqrt(d) (Appendix B).
    """
    lib = _load()
    q, k, v = _f64(q), _f64(k), _f64(v)
    q_pos, kv_pos = _i32(q_pos), _i32(kv_pos)
    tq, nh, d = q.shape
    tkv, nkv, d2 = k.shape
    assert d2 == d and v.shape == k.shape and nh % nkv == 0
    assert q_pos.shape == (tq,) and kv_pos.shape == (tkv,)
    if cu_q is None:
        assert cu_kv is None
        batch, cq, ck = 1, None, None
    else:
        cq, ck = _i32(cu_q), _i32(cu_kv)
        batch = cq.shape[0] - 1
        assert ck.shape[0] == batch + 1 and cq[-1] == tq and ck[-1] == tkv
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    out = np.empty((tq, nh, d), dtype=np.float64)
    lse = np.empty((tq, nh), dtype=np.float64)
    pairs = lib.oracle_attn(_dptr(q), _dptr(k), _dptr(v), _iptr(q_pos), _iptr(kv_pos),
                            _iptr(cq), _iptr(ck), batch, tq, tkv, nh, nkv, d,
                            float(scale), _dptr(out), _dptr(lse))
    if return_pairs:
        return out, lse, int(pairs)
    return out, lse


def merge(outs: Sequence[np.ndarray], lses: Sequence[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Equation 4 over partials outs[s] [..., d], lses[s] [...]. Returns (O, LSE)."""
    lib = _load()
    n = len(outs)
    assert n >= 1 and len(lses) == n
    o = [_f64(x) for x in outs]
    l = [_f64(x) for x in lses]
    shape = o[0].shape
    d = shape[-1]
    rows = int(np.prod(shape[:-1], dtype=np.int64))
    for a, b in zip(o, l):
        assert a.shape == shape and b.shape == shape[:-1]
    dp = ctypes.POINTER(ctypes.c_double)
    optr = (dp * n)(*[_dptr(x) for x in o])
    lptr = (dp * n)(*[_dptr(x) for x in l])
    out = np.empty(shape, dtype=np.float64)
    lse = np.empty(shape[:-1], dtype=np.float64)
    lib.oracle_merge(optr, lptr, n, rows, d, _dptr(out), _dptr(lse))
    return out, lse


def unsharded_causal(q, k, v, p_cached: int = 0, scale: Optional[float] = None):
    """Ground truth: T queries at positions P..P+T-1 against all P+T keys."""
    tq = np.asarray(q).shape[0]
    tkv = np.asarray(k).shape[0]
    assert tkv == p_cached + tq
    return attn(q, k, v, np.arange(p_cached, p_cached + tq), np.arange(tkv), scale=scale)


# --------------------------------------------------------------------------
# Section 3.5.1: load-balanced sharding
# --------------------------------------------------------------------------

def chunk_bounds(total: int, n_ranks: int) -> List[Tuple[int, int]]:
    """The 2N chunks [lo, hi) of a sequence of `total` tokens.

    Chunk size is ceil(total / 2N); trailing chunks are short or empty when
    2N does not divide the length.
    """
    n_chunks = 2 * n_ranks
    size = -(-total // n_chunks) if total > 0 else 0
    return [(min(c * size, total), min((c + 1) * size, total)) for c in range(n_chunks)]


def shard_positions(total: int, n_ranks: int, rank: int, offset: int = 0) -> np.ndarray:
    """Positions owned by `rank`: chunk `rank` then chunk 2N-1-rank, plus `offset`."""
    bounds = chunk_bounds(total, n_ranks)
    a0, a1 = bounds[rank]
    b0, b1 = bounds[2 * n_ranks - 1 - rank]
    pos = np.concatenate([np.arange(a0, a1), np.arange(b0, b1)]) + offset
    return pos.astype(np.int32)


def shard_partial_prefill(p_cached: int, t_new: int, n_ranks: int,
                          cache_partition: str = "balanced"):
    """Per-rank (q_pos, kv_pos) for partial prefill (Section 3.5.1, Figure 2).

    The T new tokens (positions P..P+T-1) are sharded load-balanced. Rank k's
    KV is its share of the cache followed by the K/V of its own new tokens.
    The cache partition is arbitrary as far as the result goes: "balanced"
    shards [0, P) with the same 2N-chunk rule, "contiguous" gives rank k the
    k-th slice.
    """
    shards = []
    for r in range(n_ranks):
        q_pos = shard_positions(t_new, n_ranks, r, offset=p_cached)
        if cache_partition == "balanced":
            c_pos = shard_positions(p_cached, n_ranks, r)
        elif cache_partition == "contiguous":
            size = -(-p_cached // n_ranks) if p_cached else 0
            c_pos = np.arange(min(r * size, p_cached), min((r + 1) * size, p_cached),
                              dtype=np.int32)
        else:
            raise ValueError(cache_partition)
        shards.append((q_pos, np.concatenate([c_pos, q_pos]).astype(np.int32)))
    return shards


def shard_decode_batch(lengths: Sequence[int], n_ranks: int, decode_iter: int = 0):
    """Placement for one batched decode step (Section 3.6, Algorithm 4).

    Sequence b has lengths[b] tokens counting the token being decoded, which
    sits at position lengths[b]-1. The lengths[b]-1 earlier tokens are sharded
    load-balanced; the new token's query and K/V belong to rank
    (b + decode_iter) mod N (round-robin, offset by one per decode iteration),
    its K/V at the end of that rank's segment for the sequence.

    Returns per rank a dict with
      kv_pos  int32 [sum_b len_{b,k}]  positions, sequences packed in order b
      kv_seq  int32 [same]             sequence id of every KV slot
      cu_kv   int32 [B+1]
      bid     int32 [n_q_k]            sequences whose query this rank owns
      q_pos   int32 [n_q_k]
    """
    n_seq = len(lengths)
    ranks = []
    for r in range(n_ranks):
        pos, seq, cu, bid, qp = [], [], [0], [], []
        for b, length in enumerate(lengths):
            p = shard_positions(length - 1, n_ranks, r)
            if (b + decode_iter) % n_ranks == r:
                p = np.concatenate([p, np.array([length - 1], dtype=np.int32)])
                bid.append(b)
                qp.append(length - 1)
            pos.append(p)
            seq.append(np.full(p.shape[0], b, dtype=np.int32))
            cu.append(cu[-1] + p.shape[0])
        ranks.append(dict(kv_pos=np.concatenate(pos).astype(np.int32),
                          kv_seq=np.concatenate(seq).astype(np.int32),
                          cu_kv=np.asarray(cu, dtype=np.int32),
                          bid=np.asarray(bid, dtype=np.int32),
                          q_pos=np.asarray(qp, dtype=np.int32)))
    assert sum(len(r["bid"]) for r in ranks) == n_seq
    return ranks


# --------------------------------------------------------------------------
# Persistent KV cache across turns (Sections 3.5.2 and 3.6)
# --------------------------------------------------------------------------

def decode_owner(seq: int, decode_iter: int, n_ranks: int) -> int:
    """Rank that takes sequence `seq`'s token at decode iteration `decode_iter` (Section 3.6:
    the batch is dealt round-robin and the deal moves on by one rank per iteration, so that
    no rank's cache grows faster than the others')."""
    return (seq + decode_iter) % n_ranks


class KVCache:
    """One rank's share of the KV cache for a batch of sequences, as plain per-sequence lists.

    Sequence b may hold at most capacity[b] tokens on this rank. `append` adds tokens of one
    sequence in order and drops (and counts) what does not fit. `packed()` lays the cache
    out as the attention functions take it: sequence b owns capacity[b] consecutive slots,
    tokens first, the unused rest carrying position INT32_MAX (never visible) and zeros.
    """

    def __init__(self, capacity: Sequence[int], n_kv_heads: int, head_dim: int):
        self.capacity = [int(c) for c in capacity]
        self.shape = (n_kv_heads, head_dim)
        self.k = [[] for _ in self.capacity]
        self.v = [[] for _ in self.capacity]
        self.pos = [[] for _ in self.capacity]
        self.dropped = 0

    def append(self, seq: int, k_new, v_new, pos_new) -> None:
        k_new = np.asarray(k_new, dtype=np.float64)
        v_new = np.asarray(v_new, dtype=np.float64)
        for i, p in enumerate(np.asarray(pos_new, dtype=np.int64)):
            if len(self.pos[seq]) >= self.capacity[seq]:
                self.dropped += 1
                continue
            self.k[seq].append(k_new[i].reshape(self.shape))
            self.v[seq].append(v_new[i].reshape(self.shape))
            self.pos[seq].append(int(p))

    def used(self) -> np.ndarray:
        return np.asarray([len(p) for p in self.pos], dtype=np.int32)

    def packed(self):
        """(k, v, kv_pos, cu_kv) with cu_kv the capacity bounds."""
        cu = np.concatenate([[0], np.cumsum(self.capacity)]).astype(np.int32)
        k = np.zeros((int(cu[-1]),) + self.shape)
        v = np.zeros_like(k)
        pos = np.full(int(cu[-1]), INT32_MAX, dtype=np.int32)
        for b in range(len(self.capacity)):
            for j in range(len(self.pos[b])):
                k[cu[b] + j] = self.k[b][j]
                v[cu[b] + j] = self.v[b][j]
                pos[cu[b] + j] = self.pos[b][j]
        return k, v, pos, cu


# --------------------------------------------------------------------------
# Algorithms 2, 3, 4: the ring, simulated over virtual ranks
# --------------------------------------------------------------------------

def ring_passkv(q, k, v, q_pos, kv_pos, scale: Optional[float] = None, cu_q=None, cu_kv=None):
    """Algorithm 2. Arguments are per-rank lists (length N). With cu_q / cu_kv (per-rank
    sequence boundaries) every rank's Q and KV are a packed batch, the fused variable-length
    input of the algorithm: a query sees the keys of its own sequence only.

    Every rank starts holding its own KV shard; at step j rank k holds the
    shard that started on rank s = (k - j) mod N, attends its queries to it,
    then takes over the previous rank's buffer. After N steps each rank merges
    its N partials locally.

    Returns (out[k], lse[k], part_out[k][s], part_lse[k][s]).
    """
    n = len(q)
    held = list(range(n))  # held[k]: origin rank of the KV buffer on rank k
    part_o = [[None] * n for _ in range(n)]
    part_l = [[None] * n for _ in range(n)]
    for j in range(n):
        for kk in range(n):
            s = (kk - j) % n
            assert held[kk] == s
            part_o[kk][s], part_l[kk][s] = attn(q[kk], k[s], v[s], q_pos[kk], kv_pos[s],
                                                cu_q=None if cu_q is None else cu_q[kk],
                                                cu_kv=None if cu_kv is None else cu_kv[s],
                                                scale=scale)
        held = [held[(kk - 1) % n] for kk in range(n)]  # receive from previous rank
    out, lse = [], []
    for kk in range(n):
        o, l = merge(part_o[kk], part_l[kk])
        out.append(o)
        lse.append(l)
    return out, lse, part_o, part_l


def ring_passq(q, k, v, q_pos, kv_pos, scale: Optional[float] = None, cu_q=None, cu_kv=None):
    """Algorithm 3. Queries circulate, KV stays. cu_q / cu_kv as in ring_passkv.

    At step j rank k holds the queries that started on rank s = (k - j) mod N
    and computes their partial output against its own KV. The partials are
    then sent back to their source rank (the permute + All2All) and merged
    there. part_out[s][k] is the partial of rank s's queries against KV_k.
    """
    n = len(q)
    held = list(range(n))
    on_rank = [[None] * n for _ in range(n)]  # on_rank[k][s]: computed on rank k for source s
    for j in range(n):
        for kk in range(n):
            s = (kk - j) % n
            assert held[kk] == s
            on_rank[kk][s] = attn(q[s], k[kk], v[kk], q_pos[s], kv_pos[kk],
                                  cu_q=None if cu_q is None else cu_q[s],
                                  cu_kv=None if cu_kv is None else cu_kv[kk], scale=scale)
        held = [held[(kk - 1) % n] for kk in range(n)]
    # All2All: source rank s receives, from every rank k, the partial computed there
    part_o = [[on_rank[kk][s][0] for kk in range(n)] for s in range(n)]
    part_l = [[on_rank[kk][s][1] for kk in range(n)] for s in range(n)]
    out, lse = [], []
    for s in range(n):
        o, l = merge(part_o[s], part_l[s])
        out.append(o)
        lse.append(l)
    return out, lse, part_o, part_l


def ring_passq_decode(q, bid, q_pos, k, v, kv_pos, cu_kv, scale: Optional[float] = None):
    """Algorithm 4. Per-rank lists: q[k] [n_q_k, N_H, d] with batch ids bid[k];
    k[k], v[k] packed KV of every sequence on rank k with boundaries cu_kv[k].

    At each step a rank attends the queries it currently holds to KV_k[bid]:
    query row r sees only the segment of sequence bid[r]. Returns
    (out[s], lse[s], part_out[s][k], part_lse[s][k]) indexed by source rank s.
    """
    n = len(q)
    held = list(range(n))
    on_rank = [[None] * n for _ in range(n)]
    for j in range(n):
        for kk in range(n):
            s = (kk - j) % n
            assert held[kk] == s
            nq = len(bid[s])
            # KV_k[bid]: gather the segments of the travelling queries' sequences
            segs = [np.arange(cu_kv[kk][b], cu_kv[kk][b + 1]) for b in bid[s]]
            idx = np.concatenate(segs) if segs else np.zeros(0, dtype=np.int64)
            cu_sel = np.concatenate([[0], np.cumsum([len(x) for x in segs])]).astype(np.int32)
            on_rank[kk][s] = attn(q[s], np.asarray(k[kk])[idx], np.asarray(v[kk])[idx],
                                  q_pos[s], np.asarray(kv_pos[kk])[idx],
                                  cu_q=np.arange(nq + 1, dtype=np.int32), cu_kv=cu_sel,
                                  scale=scale)
        held = [held[(kk - 1) % n] for kk in range(n)]
    part_o = [[on_rank[kk][s][0] for kk in range(n)] for s in range(n)]
    part_l = [[on_rank[kk][s][1] for kk in range(n)] for s in range(n)]
    out, lse = [], []
    for s in range(n):
        o, l = merge(part_o[s], part_l[s])
        out.append(o)
        lse.append(l)
    return out, lse, part_o, part_l


# ---------------------------------------------------------------------------
# pass-KV vs pass-Q (host logic)
# ---------------------------------------------------------------------------

def roofline_latencies(t_new: int, p_cached: int, n_q_heads: int, n_kv_heads: int, n_ranks: int,
                       peak_flops: float, bandwidth: float, bytes_per_elem: float = 2.0,
                       head_dim_total: float = 1.0):
    """Table 1 per ring step on N ranks: (attention, Q message, KV message, All2All) seconds.

    `head_dim_total` is D (model dimension); it multiplies every entry alike and cancels in
    every comparison, so any positive value gives the same decisions. The All2All row is
    Appendix C's (D + 1) T e / BW with the paper's D + 1 ~ D.
    """
    T, P, D, e = float(t_new), float(p_cached), float(head_dim_total), float(bytes_per_elem)
    flops = 4.0 * T * D * (T + P)
    q_bytes = T * D * e
    kv_bytes = 2.0 * (T + P) * D * (n_kv_heads / n_q_heads) * e
    attn = flops / (n_ranks * peak_flops)
    return attn, q_bytes / bandwidth, kv_bytes / bandwidth, T * D * e / bandwidth


def select_order(t_new: int, p_cached: int, n_q_heads: int, n_kv_heads: int, n_ranks: int,
                 peak_flops: float = 0.0, bandwidth: float = 0.0, bytes_per_elem: float = 2.0,
                 rule: str = "analytic", alpha: float = -1.059, beta: float = 1.145,
                 gamma: float = 12.112) -> str:
    """"pass-KV" or "pass-Q".

    analytic (Algorithm 1): pass-KV when the KV message of a ring step hides under the
    attention of that step, or when the KV message is not larger than the Q message.
    all2all (Algorithm 5): the size test is replaced by "the exposed part of the KV
    message is smaller than pass-Q's All2All of (O, LSE)".
    empirical (Appendix D): sign of alpha ln T + beta ln(T / (T + P)) + gamma; the
    paper does not say which logarithm: natural is assumed.
    """
    if rule == "empirical":
        import math
        h = alpha * math.log(t_new) + beta * math.log(t_new / (t_new + p_cached)) + gamma
        return "pass-KV" if h > 0.0 else "pass-Q"
    attn, q_msg, kv_msg, a2a = roofline_latencies(t_new, p_cached, n_q_heads, n_kv_heads,
                                                  n_ranks, peak_flops, bandwidth, bytes_per_elem)
    if attn >= kv_msg:
        return "pass-KV"
    if rule == "analytic":
        return "pass-KV" if q_msg >= kv_msg else "pass-Q"
    if rule == "all2all":
        return "pass-Q" if kv_msg - attn > a2a else "pass-KV"
    raise ValueError(rule)
