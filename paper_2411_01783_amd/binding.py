"""Thin ctypes binding of libcp_attn.so (include/cp_attn.h), same names as the C ABI.

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the path runs in the library's kernels. There is no CPU
or PyTorch fallback: a missing library raises at first use.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcp_attn.so")

CP_BF16, CP_FP32 = 0, 1
CP_WS_PARTIAL, CP_WS_DECODE, CP_WS_MERGE = 0, 1, 2
CP_POS_PAD_KV = 2**31 - 1
CP_POS_PAD_Q = -1
CP_MAX_PARTS = 64
CP_SHAPE_UNIQUE_BID = 1

EXPORTS = [
    "cp_shard_positions", "cp_workspace_bytes", "cp_attn_partial", "cp_attn_partial_accumulate",
    "cp_attn_decode", "cp_attn_decode_static",
    "cp_attn_merge", "cp_ring_passkv", "cp_ring_passq", "cp_ring_passq_decode",
    "cp_ring_workspace_bytes", "cp_ring_message_bytes", "cp_ring_prefill", "cp_select_order", "cp_kv_cache_reset", "cp_kv_append",
    "cp_decode_owner", "cp_strerror",
    "cp_version",
]
CP_STATIC_SCRATCH_BYTES = 8 << 20

_vp = ctypes.c_void_p
_i32, _i64, _f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_float


class cp_shape(ctypes.Structure):
    _fields_ = [("dtype", _i32), ("head_dim", _i32), ("n_q_heads", _i32), ("n_kv_heads", _i32),
                ("batch", _i32), ("flags", _i32), ("total_q", _i64), ("total_kv", _i64),
                ("softmax_scale", _f32), ("reserved_f", _f32)]


class cp_ring_desc(ctypes.Structure):
    _fields_ = [("dtype", _i32), ("head_dim", _i32), ("n_q_heads", _i32), ("n_kv_heads", _i32),
                ("softmax_scale", _f32), ("n_ranks", _i32), ("out_dtype", _i32),
                ("part_dtype", _i32),
                ("n_q", ctypes.POINTER(_i64)), ("n_kv", ctypes.POINTER(_i64)),
                ("q", ctypes.POINTER(_vp)), ("k", ctypes.POINTER(_vp)), ("v", ctypes.POINTER(_vp)),
                ("q_pos", ctypes.POINTER(_vp)), ("kv_pos", ctypes.POINTER(_vp)),
                ("out", ctypes.POINTER(_vp)), ("lse", ctypes.POINTER(_vp)),
                ("partial_out", _vp), ("partial_lse", _vp),
                ("keep_partials", _i32), ("fused_merge", _i32),
                ("workspace", _vp), ("workspace_bytes", ctypes.c_size_t),
                ("batch", _i32),
                ("cu_seqlens_kv", ctypes.POINTER(_vp)), ("bid", ctypes.POINTER(_vp)),
                ("aux_stream", _vp), ("message_layout", _i32),
                ("arrived", ctypes.POINTER(_vp)), ("ring_error", _vp), ("spin_limit", _i32),
                ("gathered_q", _i32), ("cu_seqlens_q", ctypes.POINTER(_vp)),
                ("unique_bid", _i32)]


class cp_select_params(ctypes.Structure):
    _fields_ = [("n_q_heads", _i32), ("n_kv_heads", _i32), ("n_ranks", _i32), ("reserved", _i32),
                ("peak_flops", ctypes.c_double), ("bandwidth", ctypes.c_double),
                ("bytes_per_elem", ctypes.c_double), ("alpha", ctypes.c_double),
                ("beta", ctypes.c_double), ("gamma", ctypes.c_double)]


CP_ORDER_PASS_KV, CP_ORDER_PASS_Q = 0, 1
CP_RULE_ANALYTIC, CP_RULE_ANALYTIC_ALL2ALL, CP_RULE_EMPIRICAL = 0, 1, 2


class CpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


_lib = None


def load() -> ctypes.CDLL:
    """Load libcp_attn.so. Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libcp_attn.so not found at %s: build it with "
            "`python -m paper_2411_01783_amd.build` (there is no CPU fallback)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    lib.cp_version.restype = ctypes.c_int
    lib.cp_strerror.restype = ctypes.c_char_p
    lib.cp_strerror.argtypes = [ctypes.c_int]
    lib.cp_shard_positions.restype = ctypes.c_int
    lib.cp_shard_positions.argtypes = [_i64, _i64, _i32, _i32, ctypes.POINTER(_i32),
                                       ctypes.POINTER(_i64)]
    lib.cp_workspace_bytes.restype = ctypes.c_size_t
    lib.cp_workspace_bytes.argtypes = [ctypes.POINTER(cp_shape), _i32]
    lib.cp_attn_partial.restype = ctypes.c_int
    lib.cp_attn_partial.argtypes = [ctypes.POINTER(cp_shape), _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                    _vp, _vp, _i32, _vp, ctypes.c_size_t, _vp]
    lib.cp_attn_decode.restype = ctypes.c_int
    lib.cp_attn_decode.argtypes = [ctypes.POINTER(cp_shape), _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                   _vp, _vp, _i32, _vp, ctypes.c_size_t, _vp]
    lib.cp_attn_decode_static.restype = ctypes.c_int
    lib.cp_attn_decode_static.argtypes = [ctypes.POINTER(cp_shape), _vp, _vp, _vp, _vp, _vp, _vp,
                                          _vp, _vp, _vp, _i32, _vp]
    lib.cp_attn_merge.restype = ctypes.c_int
    lib.cp_attn_merge.argtypes = [_i64, _i32, _i32, ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                                  _i32, _vp, _i32, _vp, _vp]
    for name in ("cp_ring_passkv", "cp_ring_passq", "cp_ring_passq_decode"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [ctypes.POINTER(cp_ring_desc), _vp]
    lib.cp_ring_workspace_bytes.restype = ctypes.c_size_t
    lib.cp_ring_workspace_bytes.argtypes = [ctypes.POINTER(cp_ring_desc), _i32]
    lib.cp_ring_prefill.restype = ctypes.c_int
    lib.cp_ring_prefill.argtypes = [ctypes.POINTER(cp_ring_desc), ctypes.POINTER(cp_select_params),
                                    _i64, _i32, ctypes.POINTER(_i32), _vp]
    lib.cp_ring_message_bytes.restype = ctypes.c_size_t
    lib.cp_ring_message_bytes.argtypes = [ctypes.POINTER(cp_ring_desc)]
    lib.cp_select_order.restype = ctypes.c_int
    lib.cp_select_order.argtypes = [ctypes.POINTER(cp_select_params), _i64, _i64, _i32,
                                    ctypes.POINTER(_i32)]
    lib.cp_attn_partial_accumulate.restype = ctypes.c_int
    lib.cp_attn_partial_accumulate.argtypes = [ctypes.POINTER(cp_shape)] + [_vp] * 8 + [_i32] + \
        [_vp] * 2 + [ctypes.c_size_t, _vp]
    lib.cp_kv_cache_reset.restype = ctypes.c_int
    lib.cp_kv_cache_reset.argtypes = [ctypes.POINTER(cp_shape)] + [_vp] * 6
    lib.cp_kv_append.restype = ctypes.c_int
    lib.cp_kv_append.argtypes = [ctypes.POINTER(cp_shape)] + [_vp] * 11
    lib.cp_decode_owner.restype = _i32
    lib.cp_decode_owner.argtypes = [_i32, _i32, _i32]
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().cp_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise CpError(status, where)


def dtype_code(dt: torch.dtype) -> int:
    if dt == torch.bfloat16:
        return CP_BF16
    if dt == torch.float32:
        return CP_FP32
    raise TypeError("unsupported dtype %s" % dt)


def torch_dtype(code: int) -> torch.dtype:
    return torch.bfloat16 if code == CP_BF16 else torch.float32


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the C ABI must be contiguous"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def make_shape(dtype: int, head_dim: int, n_q_heads: int, n_kv_heads: int, total_q: int,
               total_kv: int, batch: int = 1, softmax_scale: float = 0.0,
               flags: int = 0) -> cp_shape:
    return cp_shape(dtype, head_dim, n_q_heads, n_kv_heads, batch, flags, total_q, total_kv,
                    softmax_scale, 0.0)


# --------------------------------------------------------------------------

def cp_version() -> int:
    return int(load().cp_version())


def cp_shard_positions(total: int, n_ranks: int, rank: int, offset: int = 0) -> np.ndarray:
    """Positions owned by `rank` under load-balanced sharding (host only)."""
    lib = load()
    n = _i64(0)
    _check(lib.cp_shard_positions(total, offset, n_ranks, rank, None, ctypes.byref(n)),
           "cp_shard_positions")
    pos = np.empty(int(n.value), dtype=np.int32)
    _check(lib.cp_shard_positions(total, offset, n_ranks, rank,
                                  pos.ctypes.data_as(ctypes.POINTER(_i32)), ctypes.byref(n)),
           "cp_shard_positions")
    return pos


def cp_select_order(t_new: int, p_cached: int, n_q_heads: int, n_kv_heads: int, n_ranks: int,
                    peak_flops: float = 0.0, bandwidth: float = 0.0, bytes_per_elem: float = 2.0,
                    rule: int = CP_RULE_ANALYTIC, alpha: float = 0.0, beta: float = 0.0,
                    gamma: float = 0.0) -> int:
    """CP_ORDER_PASS_KV or CP_ORDER_PASS_Q for t_new tokens on p_cached cached (host only)."""
    prm = cp_select_params(n_q_heads, n_kv_heads, n_ranks, 0, peak_flops, bandwidth,
                           bytes_per_elem, alpha, beta, gamma)
    order = _i32(-1)
    _check(load().cp_select_order(ctypes.byref(prm), t_new, p_cached, rule, ctypes.byref(order)),
           "cp_select_order")
    return int(order.value)


def cp_workspace_bytes(shape: cp_shape, kind: int) -> int:
    return int(load().cp_workspace_bytes(ctypes.byref(shape), kind))


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes + 256, dtype=torch.uint8, device=device)


def _ws_ptr(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    p = (ws.data_ptr() + 255) & ~255
    return p, ws.numel() - (p - ws.data_ptr())


def cp_attn_partial(q, k, v, q_pos, kv_pos, cu_seqlens_q=None, cu_seqlens_kv=None,
                    out_dtype: Optional[torch.dtype] = None, softmax_scale: float = 0.0,
                    out=None, lse=None, workspace=None, stream=None):
    """(O, LSE) of q [Tq, N_H, d] against k, v [Tkv, N_KV, d] under kv_pos <= q_pos."""
    lib = load()
    tq, nh, d = q.shape
    tkv, nkv, _ = k.shape
    batch = 1 if cu_seqlens_q is None else cu_seqlens_q.numel() - 1
    shape = make_shape(dtype_code(q.dtype), d, nh, nkv, tq, tkv, batch, softmax_scale)
    odt = q.dtype if out_dtype is None else out_dtype
    if out is None:
        out = torch.empty((tq, nh, d), dtype=odt, device=q.device)
    if lse is None:
        lse = torch.empty((tq, nh), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _workspace(cp_workspace_bytes(shape, CP_WS_PARTIAL), q.device)
    wp, wn = _ws_ptr(workspace)
    _check(lib.cp_attn_partial(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(q_pos),
                               _ptr(kv_pos), _ptr(cu_seqlens_q), _ptr(cu_seqlens_kv), _ptr(out),
                               _ptr(lse), dtype_code(out.dtype), wp, wn, _stream(stream)),
           "cp_attn_partial")
    return out, lse


def cp_attn_partial_accumulate(q, k, v, q_pos, kv_pos, acc_out, acc_lse, final_out=None,
                               final_lse=None, softmax_scale: float = 0.0, workspace=None,
                               stream=None):
    """Merge Attn(q, kv) into the running fp32 (acc_out, acc_lse); see the header."""
    lib = load()
    tq, nh, d = q.shape
    tkv, nkv, _ = k.shape
    shape = make_shape(dtype_code(q.dtype), d, nh, nkv, tq, tkv, 1, softmax_scale)
    assert acc_out.dtype == torch.float32 and acc_lse.dtype == torch.float32
    if workspace is None:
        workspace = _workspace(cp_workspace_bytes(shape, CP_WS_PARTIAL), q.device)
    wp, wn = _ws_ptr(workspace)
    fdt = dtype_code(final_out.dtype) if final_out is not None else CP_FP32
    _check(lib.cp_attn_partial_accumulate(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v),
                                          _ptr(q_pos), _ptr(kv_pos), _ptr(acc_out), _ptr(acc_lse),
                                          _ptr(final_out), fdt, _ptr(final_lse), wp, wn,
                                          _stream(stream)), "cp_attn_partial_accumulate")
    return (final_out if final_out is not None else acc_out), acc_lse


def cp_attn_decode(q, k, v, q_pos, kv_pos, cu_seqlens_kv, bid,
                   out_dtype: Optional[torch.dtype] = None, softmax_scale: float = 0.0,
                   out=None, lse=None, workspace=None, stream=None, unique_bid: bool = False):
    """Decode step: query i attends to KV segment bid[i] of the packed k, v. `unique_bid`:
    the caller's promise that no sequence id occurs twice (CP_SHAPE_UNIQUE_BID)."""
    lib = load()
    nq, nh, d = q.shape
    tkv, nkv, _ = k.shape
    batch = cu_seqlens_kv.numel() - 1
    shape = make_shape(dtype_code(q.dtype), d, nh, nkv, nq, tkv, batch, softmax_scale,
                       CP_SHAPE_UNIQUE_BID if unique_bid else 0)
    odt = q.dtype if out_dtype is None else out_dtype
    if out is None:
        out = torch.empty((nq, nh, d), dtype=odt, device=q.device)
    if lse is None:
        lse = torch.empty((nq, nh), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _workspace(cp_workspace_bytes(shape, CP_WS_DECODE), q.device)
    wp, wn = _ws_ptr(workspace)
    _check(lib.cp_attn_decode(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(q_pos),
                              _ptr(kv_pos), _ptr(cu_seqlens_kv), _ptr(bid), _ptr(out), _ptr(lse),
                              dtype_code(out.dtype), wp, wn, _stream(stream)),
           "cp_attn_decode")
    return out, lse


def cp_attn_decode_static(q, k, v, q_pos, kv_pos, cu_seqlens_kv, bid, out, lse,
                          softmax_scale: float = 0.0, stream=None, unique_bid: bool = False):
    """cp_attn_decode into caller-provided `out` / `lse`, with the library's own scratch array
    in place of a workspace: the call allocates nothing (nor does this wrapper)."""
    nq, nh, d = q.shape
    tkv, nkv, _ = k.shape
    shape = make_shape(dtype_code(q.dtype), d, nh, nkv, nq, tkv, cu_seqlens_kv.numel() - 1,
                       softmax_scale, CP_SHAPE_UNIQUE_BID if unique_bid else 0)
    _check(load().cp_attn_decode_static(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v),
                                        _ptr(q_pos), _ptr(kv_pos), _ptr(cu_seqlens_kv), _ptr(bid),
                                        _ptr(out), _ptr(lse), dtype_code(out.dtype),
                                        _stream(stream)), "cp_attn_decode_static")
    return out, lse


class KVCache:
    """Device buffers of one rank's persistent KV cache (see cp_kv_append in cp_attn.h):
    a holder for the tensors, nothing else. `capacity[b]` slots per sequence."""

    def __init__(self, capacity: Sequence[int], n_kv_heads: int, head_dim: int,
                 dtype: torch.dtype = torch.bfloat16, device="cuda", stream=None):
        cu = np.concatenate([[0], np.cumsum(np.asarray(capacity, dtype=np.int64))])
        self.batch = len(capacity)
        self.slots = int(cu[-1])
        self.cu_host = cu.astype(np.int32)
        self.cu = torch.as_tensor(self.cu_host).to(device)
        self.k = torch.empty((self.slots, n_kv_heads, head_dim), dtype=dtype, device=device)
        self.v = torch.empty_like(self.k)
        self.kv_pos = torch.empty((self.slots,), dtype=torch.int32, device=device)
        self.used = torch.empty((self.batch + 1,), dtype=torch.int32, device=device)  # + ticket word
        self.dropped = torch.empty((1,), dtype=torch.int32, device=device)
        shape = make_shape(dtype_code(dtype), head_dim, n_kv_heads, n_kv_heads, 0, self.slots,
                           self.batch)
        _check(load().cp_kv_cache_reset(ctypes.byref(shape), _ptr(self.k), _ptr(self.v),
                                        _ptr(self.kv_pos), _ptr(self.used), _ptr(self.dropped),
                                        _stream(stream)), "cp_kv_cache_reset")

    def segment(self, b: int):
        """(k, v, kv_pos) views of sequence b's slot range, unused slots included."""
        lo, hi = int(self.cu_host[b]), int(self.cu_host[b + 1])
        return self.k[lo:hi], self.v[lo:hi], self.kv_pos[lo:hi]


def cp_kv_append(cache: KVCache, k_new: torch.Tensor, v_new: torch.Tensor,
                 pos_new: torch.Tensor, cu_seqlens_new: torch.Tensor, stream=None) -> None:
    """Append rows [cu_new[b], cu_new[b+1]) of k_new / v_new to sequence b of the cache."""
    n_new, nkv, d = k_new.shape
    shape = make_shape(dtype_code(k_new.dtype), d, nkv, nkv, n_new, cache.slots, cache.batch)
    if k_new.dtype != cache.k.dtype or tuple(cache.k.shape[1:]) != (nkv, d):
        raise ValueError("new K/V rows do not match the cache's row shape or dtype")
    if cu_seqlens_new.numel() != cache.batch + 1 or pos_new.numel() != n_new:
        raise ValueError("cu_seqlens_new / pos_new sizes do not match")
    _check(load().cp_kv_append(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(pos_new),
                               _ptr(cu_seqlens_new), _ptr(cache.k), _ptr(cache.v),
                               _ptr(cache.kv_pos), _ptr(cache.cu), _ptr(cache.used),
                               _ptr(cache.dropped), _stream(stream)), "cp_kv_append")


def cp_decode_owner(seq: int, decode_iter: int, n_ranks: int) -> int:
    r = int(load().cp_decode_owner(seq, decode_iter, n_ranks))
    _check(min(r, 0), "cp_decode_owner")
    return r


def cp_attn_merge(outs: Sequence[torch.Tensor], lses: Sequence[torch.Tensor],
                  out_dtype: Optional[torch.dtype] = None, out=None, lse_out=None,
                  want_lse: bool = True, stream=None):
    """Equation 4 over partial outputs outs[s] [..., d] with lses[s] [...]."""
    lib = load()
    n = len(outs)
    d = outs[0].shape[-1]
    rows = outs[0].numel() // d
    odt = outs[0].dtype if out_dtype is None else out_dtype
    if out is None:
        out = torch.empty(outs[0].shape, dtype=odt, device=outs[0].device)
    if lse_out is None and want_lse:
        lse_out = torch.empty(outs[0].shape[:-1], dtype=torch.float32, device=outs[0].device)
    optr = (_vp * n)(*[_ptr(t) for t in outs])
    lptr = (_vp * n)(*[_ptr(t) for t in lses])
    _check(lib.cp_attn_merge(rows, d, n, optr, lptr, dtype_code(outs[0].dtype), _ptr(out),
                             dtype_code(out.dtype), _ptr(lse_out), _stream(stream)),
           "cp_attn_merge")
    return out, lse_out


class Ring:
    """Owns the host-side arrays of a cp_ring_desc and the device scratch it points to."""

    def __init__(self, q: List[torch.Tensor], k: List[torch.Tensor], v: List[torch.Tensor],
                 q_pos: List[torch.Tensor], kv_pos: List[torch.Tensor],
                 out_dtype: Optional[torch.dtype] = None, part_dtype: torch.dtype = torch.float32,
                 keep_partials: bool = False, softmax_scale: float = 0.0,
                 cu_seqlens_kv: Optional[List[torch.Tensor]] = None,
                 bid: Optional[List[torch.Tensor]] = None, aux_stream=None,
                 fused_merge=False, message_layout: bool = False,
                 arrived: Optional[List[torch.Tensor]] = None, spin_limit: int = 1 << 16,
                 gathered_q: bool = False,
                 cu_seqlens_q: Optional[List[torch.Tensor]] = None, unique_bid: bool = False):
        n = len(q)
        self.n = n
        self.decode = cu_seqlens_kv is not None and cu_seqlens_q is None
        dev = q[0].device
        _, nh, d = q[0].shape
        nkv = k[0].shape[1]
        odt = q[0].dtype if out_dtype is None else out_dtype
        self.tensors = (q, k, v, q_pos, kv_pos, cu_seqlens_kv, bid)  # keep alive
        self.n_q = [int(t.shape[0]) for t in q]
        self.n_kv = [int(t.shape[0]) for t in k]
        if gathered_q:   # outputs back to back like the queries: one merge launch for all ranks
            tot = sum(self.n_q)
            self.out_all = torch.empty((tot, nh, d), dtype=odt, device=dev)
            self.lse_all = torch.empty((tot, nh), dtype=torch.float32, device=dev)
            ends = np.cumsum([0] + self.n_q)
            self.out = [self.out_all[ends[i]:ends[i + 1]] for i in range(n)]
            self.lse = [self.lse_all[ends[i]:ends[i + 1]] for i in range(n)]
        else:
            self.out = [torch.empty((m, nh, d), dtype=odt, device=dev) for m in self.n_q]
            self.lse = [torch.empty((m, nh), dtype=torch.float32, device=dev) for m in self.n_q]
        max_q = max(self.n_q) if self.n_q else 0
        slots = n * n if keep_partials else (1 if fused_merge else n)
        self.keep = keep_partials
        self.messages = None
        if not message_layout:
            self.partial_out = torch.empty((slots, max_q, nh, d), dtype=part_dtype, device=dev)
            self.partial_lse = torch.empty((slots, max_q, nh), dtype=torch.float32, device=dev)

        def parr(ts):
            return (_vp * n)(*[(_ptr(t) if t is not None and t.numel() > 0 else None) for t in ts])

        self._arrs = dict(
            n_q=(_i64 * n)(*self.n_q), n_kv=(_i64 * n)(*self.n_kv),
            q=parr(q), k=parr(k), v=parr(v), q_pos=parr(q_pos), kv_pos=parr(kv_pos),
            out=parr(self.out), lse=parr(self.lse))
        dsc = cp_ring_desc()
        dsc.dtype, dsc.head_dim, dsc.n_q_heads, dsc.n_kv_heads = dtype_code(q[0].dtype), d, nh, nkv
        dsc.softmax_scale, dsc.n_ranks = softmax_scale, n
        dsc.out_dtype, dsc.part_dtype = dtype_code(odt), dtype_code(part_dtype)
        for name, arr in self._arrs.items():
            setattr(dsc, name, ctypes.cast(arr, type(getattr(dsc, name))))
        if message_layout:
            # one buffer of messages (O of the slot, then its LSE), see cp_ring_desc
            dsc.message_layout = 1
            self.message_bytes = int(load().cp_ring_message_bytes(ctypes.byref(dsc)))
            self.messages = torch.empty((slots, self.message_bytes), dtype=torch.uint8,
                                        device=dev)
            o_bytes = max_q * nh * d * torch.empty(0, dtype=part_dtype).element_size()
            self.partial_out = self.messages[:, :o_bytes].view(part_dtype).view(slots, max_q, nh, d)
            self.partial_lse = self.messages[:, o_bytes:o_bytes + max_q * nh * 4] \
                .view(torch.float32).view(slots, max_q, nh)
            dsc.partial_out, dsc.partial_lse = _ptr(self.messages), None
        else:
            dsc.partial_out, dsc.partial_lse = _ptr(self.partial_out), _ptr(self.partial_lse)
        dsc.keep_partials = 1 if keep_partials else 0
        dsc.fused_merge = int(fused_merge)   # False/True, or 2: all steps of a rank in one launch
        dsc.gathered_q = 1 if gathered_q else 0
        dsc.unique_bid = 1 if unique_bid else 0
        self.gathered = gathered_q
        self.arrived = arrived
        if arrived is not None:
            self._arrived = (_vp * n)(*[_ptr(t) for t in arrived])
            dsc.arrived = ctypes.cast(self._arrived, ctypes.POINTER(_vp))
            self.ring_error = torch.zeros(n, dtype=torch.int32, device=dev)   # per rank: bit j = step j
            dsc.ring_error = _ptr(self.ring_error)
            dsc.spin_limit = spin_limit
        if cu_seqlens_q is not None:   # packed prefill batch
            self._cuq = (_vp * n)(*[_ptr(t) for t in cu_seqlens_q])
            self._cu = (_vp * n)(*[_ptr(t) for t in cu_seqlens_kv])
            dsc.batch = cu_seqlens_q[0].numel() - 1
            dsc.cu_seqlens_q = ctypes.cast(self._cuq, ctypes.POINTER(_vp))
            dsc.cu_seqlens_kv = ctypes.cast(self._cu, ctypes.POINTER(_vp))
            self.tensors = self.tensors + (cu_seqlens_q,)
        if self.decode:
            self._cu = (_vp * n)(*[_ptr(t) for t in cu_seqlens_kv])
            self._bid = (_vp * n)(*[(_ptr(t) if t.numel() > 0 else None) for t in bid])
            dsc.batch = cu_seqlens_kv[0].numel() - 1
            dsc.cu_seqlens_kv = ctypes.cast(self._cu, ctypes.POINTER(_vp))
            dsc.bid = ctypes.cast(self._bid, ctypes.POINTER(_vp))
        self.aux_stream = aux_stream  # keep alive
        if aux_stream is not None:
            dsc.aux_stream = aux_stream.cuda_stream
        self.desc = dsc
        nbytes = int(load().cp_ring_workspace_bytes(ctypes.byref(dsc), 1 if self.decode else 0))
        self.workspace = _workspace(nbytes, dev)
        wp, wn = _ws_ptr(self.workspace)
        dsc.workspace, dsc.workspace_bytes = wp, wn

    def arrival_failed(self) -> bool:
        """True if a ring walk gave up waiting for a shard (synchronises the device)."""
        if self.arrived is None:
            return False
        torch.cuda.synchronize()
        return bool((self.ring_error != 0).any().item())

    def partial(self, a: int, b: int):
        """Partial (O, LSE) of rank a's queries against rank b's KV (keep_partials only)."""
        assert self.keep
        m = self.n_q[a]
        slot = b * self.n + a if self.gathered else a * self.n + b
        return self.partial_out[slot, :m], self.partial_lse[slot, :m]


def cp_ring_passkv(ring: Ring, stream=None):
    _check(load().cp_ring_passkv(ctypes.byref(ring.desc), _stream(stream)), "cp_ring_passkv")
    return ring.out, ring.lse


def cp_ring_passq(ring: Ring, stream=None):
    _check(load().cp_ring_passq(ctypes.byref(ring.desc), _stream(stream)), "cp_ring_passq")
    return ring.out, ring.lse


def cp_ring_prefill(ring: Ring, p_cached: int, n_q_heads: int, n_kv_heads: int,
                    peak_flops: float, bandwidth: float, bytes_per_elem: float = 2.0,
                    rule: int = CP_RULE_ANALYTIC, stream=None):
    """Prefill in the order cp_select_order picks; returns (out, lse, order)."""
    prm = cp_select_params(n_q_heads, n_kv_heads, ring.n, 0, peak_flops, bandwidth,
                           bytes_per_elem, 0.0, 0.0, 0.0)
    order = _i32(-1)
    _check(load().cp_ring_prefill(ctypes.byref(ring.desc), ctypes.byref(prm), p_cached, rule,
                                  ctypes.byref(order), _stream(stream)), "cp_ring_prefill")
    return ring.out, ring.lse, int(order.value)


def cp_ring_passq_decode(ring: Ring, stream=None):
    _check(load().cp_ring_passq_decode(ctypes.byref(ring.desc), _stream(stream)),
           "cp_ring_passq_decode")
    return ring.out, ring.lse
