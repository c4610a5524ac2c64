"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, validates arguments before touching a device, and its sharding
function agrees with the oracle's."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2411_01783_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2411_01783_amd import build
        build.build()
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "cp_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(cp_[a-z_0-9]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_partial_accumulate_rejects_what_it_cannot_run(lib):
    import ctypes
    one = ctypes.c_void_p(256)  # never dereferenced: every call below fails validation first
    def call(shape):
        return lib.cp_attn_partial_accumulate(ctypes.byref(shape), one, one, one, one, one, one, one,
                                              None, 0, None, one, ctypes.c_size_t(1 << 30), None)
    # fp32 inputs, head_dim 64, a packed batch, and a query shard short enough to split the KV axis
    assert call(B.make_shape(B.CP_FP32, 128, 16, 1, 4096, 4096)) == -3
    assert call(B.make_shape(B.CP_BF16, 64, 16, 1, 4096, 4096)) == -3
    assert call(B.make_shape(B.CP_BF16, 128, 16, 1, 4096, 4096, batch=2)) == -3
    assert call(B.make_shape(B.CP_BF16, 128, 16, 1, 64, 4096)) == -3
    ok_shape = B.make_shape(B.CP_BF16, 128, 16, 1, 4096, 4096)
    assert lib.cp_attn_partial_accumulate(ctypes.byref(ok_shape), one, one, one, one, one, None, one,
                                          None, 0, None, one, ctypes.c_size_t(1 << 30), None) == -1


def test_kv_cache_calls_validate_before_launching(lib):
    one = ctypes.c_void_p(256)    # never dereferenced: every call below fails validation first
    odd = ctypes.c_void_p(264)    # not 16-byte aligned
    def reset(shape, k_cache=one, used=one):
        return lib.cp_kv_cache_reset(ctypes.byref(shape), k_cache, one, one, used, None, None)
    assert reset(B.make_shape(B.CP_BF16, 128, 1, 1, 0, -1, batch=2)) == -2
    assert reset(B.make_shape(B.CP_BF16, 128, 1, 1, 0, 2 ** 31, batch=2)) == -2
    assert reset(B.make_shape(B.CP_BF16, 128, 1, 1, 0, 64, batch=0)) == -2
    assert reset(B.make_shape(B.CP_BF16, 12, 1, 1, 0, 64, batch=2)) == -3
    assert reset(B.make_shape(B.CP_BF16, 128, 1, 1, 0, 64, batch=2), k_cache=None) == -1
    assert reset(B.make_shape(B.CP_BF16, 128, 1, 1, 0, 64, batch=2), used=None) == -1
    assert reset(B.make_shape(B.CP_BF16, 128, 1, 1, 0, 64, batch=2), k_cache=odd) == -6

    def call(shape, k_new=one, cu_new=one, used=one, k_cache=one):
        return lib.cp_kv_append(ctypes.byref(shape), k_new, one, one, cu_new, k_cache, one, one,
                                one, used, None, None)
    good = B.make_shape(B.CP_BF16, 128, 1, 1, 4, 64, batch=2)
    assert call(good, k_new=None) == -1
    assert call(good, cu_new=None) == -1
    assert call(good, used=None) == -1
    assert call(good, k_cache=odd) == -6
    assert call(B.make_shape(7, 128, 1, 1, 4, 64, batch=2)) == -3
    assert call(B.make_shape(B.CP_BF16, 100, 1, 1, 4, 64, batch=2)) == -3
    assert call(B.make_shape(B.CP_BF16, 128, 1, 1, 4, 64, batch=0)) == -2
    assert call(B.make_shape(B.CP_BF16, 128, 1, 1, -4, 64, batch=2)) == -2
    # nothing to append: accepted without touching any buffer
    assert call(B.make_shape(B.CP_BF16, 128, 1, 1, 0, 64, batch=2), k_new=None) == 0


def test_decode_owner_matches_oracle(lib, oracle):
    for n in (1, 3, 16):
        for b in range(7):
            for t in range(5):
                assert lib.cp_decode_owner(b, t, n) == oracle.decode_owner(b, t, n)
    assert lib.cp_decode_owner(0, 0, 0) == -2
    assert lib.cp_decode_owner(-1, 0, 4) == -2


def test_ring_prefill_validates_before_launching(lib):
    d = B.cp_ring_desc()
    prm = B.cp_select_params(128, 8, 4, 0, 1e15, 5e10, 2.0, 0.0, 0.0, 0.0)
    order = ctypes.c_int32(-1)
    assert lib.cp_ring_prefill(None, ctypes.byref(prm), 0, 0, ctypes.byref(order), None) == -1
    assert lib.cp_ring_prefill(ctypes.byref(d), None, 0, 0, ctypes.byref(order), None) == -1
    d.n_ranks = 4
    assert lib.cp_ring_prefill(ctypes.byref(d), ctypes.byref(prm), 0, 0, None, None) == -2  # n_q
    n_q = (ctypes.c_int64 * 4)(0, 0, 0, 0)
    d.n_q = ctypes.cast(n_q, type(d.n_q))
    assert lib.cp_ring_prefill(ctypes.byref(d), ctypes.byref(prm), 0, 0, None, None) == -2  # T = 0
    n_q[0] = 16
    prm.n_ranks = 8
    assert lib.cp_ring_prefill(ctypes.byref(d), ctypes.byref(prm), 0, 0, None, None) == -2
    prm.n_ranks = 4
    assert lib.cp_ring_prefill(ctypes.byref(d), ctypes.byref(prm), 0, 9, None, None) == -3  # rule
    # a valid choice, then the driver's own validation (the descriptor has no arrays)
    assert lib.cp_ring_prefill(ctypes.byref(d), ctypes.byref(prm), 0, 0, ctypes.byref(order),
                               None) == -1
    assert order.value == B.CP_ORDER_PASS_KV


def test_version_and_strerror(lib):
    assert B.cp_version() >= 100
    assert B.strerror(0) == "ok"
    for code in range(-6, 0):
        assert B.strerror(code) not in ("ok", "unknown status")
    assert B.strerror(-99) == "unknown status"


@pytest.mark.parametrize("total,n", [(512, 2), (131072, 16), (37, 3), (5, 4), (1, 2), (0, 2),
                                     (64, 1), (1000, 16), (4095, 16)])
def test_shard_positions_matches_oracle(lib, oracle, total, n):
    for rank in range(n):
        for offset in (0, 131072):
            got = B.cp_shard_positions(total, n, rank, offset)
            want = oracle.shard_positions(total, n, rank, offset)
            np.testing.assert_array_equal(got, want)


def test_shard_positions_rejects_bad_arguments(lib):
    n = ctypes.c_int64(0)
    f = lib.cp_shard_positions
    assert f(10, 0, 2, 0, None, None) == -1
    assert f(-1, 0, 2, 0, None, ctypes.byref(n)) == -2
    assert f(10, 0, 0, 0, None, ctypes.byref(n)) == -2
    assert f(10, 0, 2, 2, None, ctypes.byref(n)) == -2
    assert f(10, -1, 2, 0, None, ctypes.byref(n)) == -2
    assert f(2**31, 0, 2, 0, None, ctypes.byref(n)) == -2


def _shape(**kw):
    base = dict(dtype=B.CP_BF16, head_dim=128, n_q_heads=16, n_kv_heads=1, total_q=64,
                total_kv=256, batch=1, softmax_scale=0.0)
    base.update(kw)
    return B.make_shape(**base)


def _partial(lib, shape, q=0x1000, k=0x1000, v=0x1000, qp=0x1000, kp=0x1000, cq=None, ck=None,
             out=0x1000, lse=0x1000, odt=B.CP_FP32, ws=0x1000, wsn=1 << 40):
    return lib.cp_attn_partial(ctypes.byref(shape), q, k, v, qp, kp, cq, ck, out, lse, odt, ws,
                               wsn, None)


def test_partial_validates_before_launching(lib):
    # none of these may reach the device: the fake pointers would fault if dereferenced
    assert lib.cp_attn_partial(None, 1, 1, 1, 1, 1, None, None, 1, 1, 0, None, 0, None) == -1
    assert _partial(lib, _shape(head_dim=96)) == -3
    assert _partial(lib, _shape(dtype=7)) == -3
    assert _partial(lib, _shape(n_q_heads=6, n_kv_heads=4)) == -2
    assert _partial(lib, _shape(n_kv_heads=0)) == -2
    assert _partial(lib, _shape(total_q=-1)) == -2
    assert _partial(lib, _shape(batch=0)) == -2
    assert _partial(lib, _shape(batch=2)) == -2           # batch > 1 without cu_seqlens
    assert _partial(lib, _shape(softmax_scale=float("nan"))) == -2
    assert _partial(lib, _shape(), q=None) == -1
    assert _partial(lib, _shape(), kp=None) == -1
    assert _partial(lib, _shape(), lse=None) == -1
    assert _partial(lib, _shape(), cq=0x1000) == -1       # only one of the two cu_seqlens
    assert _partial(lib, _shape(), odt=5) == -3
    assert _partial(lib, _shape(), k=0x1008) == -6
    assert _partial(lib, _shape(), ws=None) == -4
    assert _partial(lib, _shape(), ws=0x1010) == -4       # not 256-byte aligned
    assert _partial(lib, _shape(), wsn=16) == -4
    assert _partial(lib, _shape(total_q=0)) == 0          # nothing to do, nothing launched
    s = _shape()
    s.flags = 2
    assert _partial(lib, s) == -2


def test_decode_validates_before_launching(lib):
    def dec(shape, cu=0x1000, bid=0x1000, ws=0x1000, wsn=1 << 40, q=0x1000):
        return lib.cp_attn_decode(ctypes.byref(shape), q, 0x1000, 0x1000, 0x1000, 0x1000, cu, bid,
                                  0x1000, 0x1000, B.CP_FP32, ws, wsn, None)
    assert dec(_shape(dtype=B.CP_FP32)) == -3
    assert dec(_shape(head_dim=64)) == -3
    assert dec(_shape(n_q_heads=32)) == -3                # group of 32 > 16
    assert dec(_shape(), cu=None) == -1
    assert dec(_shape(), bid=None) == -1
    assert dec(_shape(), ws=None) == -4
    assert dec(_shape(), wsn=8) == -4
    assert dec(_shape(), q=0x1004) == -6
    assert dec(_shape(total_q=0)) == 0


def test_decode_static_rejects_what_does_not_fit(lib):
    # 4096 queries x 16 heads x 2+ splits of fp32 partials is far beyond the scratch array
    shape = B.make_shape(B.CP_BF16, 128, 16, 1, 4096, 4096 * 4096, batch=4096)
    assert B.cp_workspace_bytes(shape, B.CP_WS_DECODE) > B.CP_STATIC_SCRATCH_BYTES
    one = ctypes.c_void_p(256)
    rc = lib.cp_attn_decode_static(ctypes.byref(shape), one, one, one, one, one, one, one, one,
                                   one, B.CP_FP32, None)
    assert rc == -4   # CP_ERR_WORKSPACE, before anything is launched


def test_merge_validates_before_launching(lib):
    vp = ctypes.c_void_p

    def mrg(rows=8, d=128, n=2, outs=(0x1000, 0x2000), lses=(0x1000, 0x2000), pdt=B.CP_FP32,
            out=0x1000, odt=B.CP_BF16):
        o = (vp * len(outs))(*outs) if outs is not None else None
        l = (vp * len(lses))(*lses) if lses is not None else None
        return lib.cp_attn_merge(rows, d, n, o, l, pdt, out, odt, None, None)
    assert mrg(rows=-1) == -2
    assert mrg(d=12) == -2
    assert mrg(d=512) == -2
    assert mrg(n=0) == -2
    assert mrg(n=65, outs=(0x1000,) * 65, lses=(0x1000,) * 65) == -2
    assert mrg(pdt=3) == -3
    assert mrg(outs=None) == -1
    assert mrg(outs=(0x1000, None)) == -1
    assert mrg(out=None) == -1
    assert mrg(outs=(0x1000, 0x2004)) == -6
    assert mrg(rows=0) == 0


def test_workspace_sizes(lib):
    # long query shard: only the per-tile position bounds (8 bytes per 128 keys)
    big = _shape(total_q=8192, total_kv=8192)
    assert B.cp_workspace_bytes(big, B.CP_WS_PARTIAL) == 64 * 8
    # short query shard: split over KV, fp32 partial O and LSE per split
    small = _shape(total_q=64, total_kv=8256)
    n = B.cp_workspace_bytes(small, B.CP_WS_PARTIAL)
    assert n > 64 * 16 * 128 * 4
    # shapes the vector kernel serves need none
    assert B.cp_workspace_bytes(_shape(dtype=B.CP_FP32, head_dim=64), B.CP_WS_PARTIAL) == 0
    assert B.cp_workspace_bytes(_shape(head_dim=96), B.CP_WS_PARTIAL) == 0
    dec = _shape(total_q=32, total_kv=163840, batch=32)
    assert B.cp_workspace_bytes(dec, B.CP_WS_DECODE) >= 32 * 16 * 128 * 4
    assert B.cp_workspace_bytes(dec, B.CP_WS_MERGE) == 0


def test_ring_descriptor_validation(lib):
    d = B.cp_ring_desc()
    assert lib.cp_ring_passkv(None, None) == -1
    d.n_ranks = 0
    assert lib.cp_ring_passkv(ctypes.byref(d), None) == -2
    d.n_ranks = 2
    assert lib.cp_ring_passkv(ctypes.byref(d), None) == -1   # per-rank arrays missing
    assert lib.cp_ring_passq(ctypes.byref(d), None) == -1
    assert lib.cp_ring_passq_decode(ctypes.byref(d), None) == -1
    assert lib.cp_ring_workspace_bytes(ctypes.byref(d), 0) == 0
    d.message_layout = 2
    assert lib.cp_ring_passkv(ctypes.byref(d), None) == -2
    d.message_layout = 0
    d.fused_merge = 3
    assert lib.cp_ring_passkv(ctypes.byref(d), None) == -2
    d.fused_merge = 0


def test_ring_message_bytes(lib):
    d = B.cp_ring_desc()
    assert lib.cp_ring_message_bytes(None) == 0
    assert lib.cp_ring_message_bytes(ctypes.byref(d)) == 0      # no ranks
    n_q = (ctypes.c_int64 * 3)(5, 8192, 100)
    d.n_ranks, d.n_q_heads, d.head_dim, d.part_dtype = 3, 16, 128, B.CP_BF16
    d.n_q = ctypes.cast(n_q, type(d.n_q))
    # O of the largest shard (D elements a row) and its LSE (one float a row), to 256 bytes:
    # Appendix C's (D + 1) per row with the LSE kept in fp32
    rows = 8192 * 16
    assert lib.cp_ring_message_bytes(ctypes.byref(d)) == rows * 128 * 2 + rows * 4
    d.part_dtype = B.CP_FP32
    assert lib.cp_ring_message_bytes(ctypes.byref(d)) == rows * (128 + 1) * 4
    n_q[1] = 7
    assert lib.cp_ring_message_bytes(ctypes.byref(d)) == -(-(100 * 16 * 129 * 4) // 256) * 256
    d.part_dtype = 9
    assert lib.cp_ring_message_bytes(ctypes.byref(d)) == 0


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2411_01783_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "cp_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2411_01783_amd" not in text and "cp_attn.h" not in text, f


def test_select_order_matches_oracle(lib, oracle):
    names = {B.CP_ORDER_PASS_KV: "pass-KV", B.CP_ORDER_PASS_Q: "pass-Q"}
    rules = {B.CP_RULE_ANALYTIC: "analytic", B.CP_RULE_ANALYTIC_ALL2ALL: "all2all",
             B.CP_RULE_EMPIRICAL: "empirical"}
    rng = np.random.default_rng(7)
    for _ in range(400):
        t = int(rng.integers(1, 200_000))
        p = int(rng.integers(0, 2_000_000))
        nkv = int(rng.choice([1, 2, 8]))
        nh = nkv * int(rng.choice([1, 2, 4, 16]))
        n = int(rng.choice([1, 2, 4, 8, 16]))
        c = float(rng.uniform(1e14, 3e15))
        bw = float(rng.uniform(1e10, 1e12))
        for rule, rname in rules.items():
            got = B.cp_select_order(t, p, nh, nkv, n, c, bw, 2.0, rule)
            want = oracle.select_order(t, p, nh, nkv, n, c, bw, 2.0, rname)
            assert names[got] == want, (t, p, nh, nkv, n, c, bw, rname)


def test_select_order_rejects_bad_arguments(lib):
    prm = B.cp_select_params(16, 1, 4, 0, 1e15, 1e11, 2.0, 0.0, 0.0, 0.0)
    out = ctypes.c_int32(-1)
    f = lib.cp_select_order
    assert f(None, 1, 0, 0, ctypes.byref(out)) == -1
    assert f(ctypes.byref(prm), 1, 0, 0, None) == -1
    assert f(ctypes.byref(prm), 0, 0, 0, ctypes.byref(out)) == -2
    assert f(ctypes.byref(prm), 1, -1, 0, ctypes.byref(out)) == -2
    assert f(ctypes.byref(prm), 1, 0, 9, ctypes.byref(out)) == -3
    bad = B.cp_select_params(16, 1, 4, 0, 0.0, 1e11, 2.0, 0.0, 0.0, 0.0)
    assert f(ctypes.byref(bad), 1, 0, 0, ctypes.byref(out)) == -2
    assert f(ctypes.byref(bad), 1, 0, 2, ctypes.byref(out)) == 0   # empirical rule needs no C / BW


def test_ctypes_structs_match_the_header_layout(tmp_path):
    """The binding's ctypes mirrors of cp_shape, cp_ring_desc and cp_select_params have the
    size and field offsets the C compiler gives the header's structs."""
    import subprocess
    structs = {"cp_shape": B.cp_shape, "cp_ring_desc": B.cp_ring_desc,
               "cp_select_params": B.cp_select_params}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "cp_attn.h"', 'int main(void) {']
    for name, cls in structs.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (name, name))
        for field, _ in cls._fields_:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (name, field, name, field))
    lines += ['return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o",
                    str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    got = dict(line.split() for line in out.strip().splitlines())
    for name, cls in structs.items():
        assert int(got[name]) == ctypes.sizeof(cls), name
        for field, _ in cls._fields_:
            assert int(got["%s.%s" % (name, field)]) == getattr(cls, field).offset, (name, field)


def test_bench_probe_library_builds_and_validates():
    """bench.py's yardstick kernels live in a library of their own, outside the C ABI."""
    from bench_support import probes
    probes.build()
    lib = probes.load()
    flop = ctypes.c_double(0.0)
    one = ctypes.c_void_p(256)  # never dereferenced: every call below fails validation first
    assert lib.bench_probe_mfma_rate(None, 1, 1, one, ctypes.byref(flop), None) == -1
    assert lib.bench_probe_mfma_rate(one, 0, 1, one, ctypes.byref(flop), None) == -2
    assert lib.bench_probe_hbm_read(None, ctypes.c_size_t(1024), 1, one, None) == -1
    assert lib.bench_probe_hbm_read(one, ctypes.c_size_t(1000), 1, one, None) == -2
    assert lib.bench_probe_hbm_read(ctypes.c_void_p(260), ctypes.c_size_t(1024), 1, one, None) == -6
    assert not hasattr(B.load(), "cp_probe_mfma_rate")
