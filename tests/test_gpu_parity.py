"""GPU parity: every entry point of the C-ABI library against the fp64 oracle, element by
element on the same seeded inputs, at sizes the oracle finishes in seconds that still span
several tiles and ragged tails. All calls go through the ctypes binding of the C ABI."""
import numpy as np
import pytest
import torch

from gpu_util import (LSE_RTOL_FP32, O_ATOL_FP32, check, dev, i32, randn)
from paper_2411_01783_amd import binding as B
from paper_2411_01783_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    B.load()  # raises if the HIP library is missing: no fallback
    assert torch.cuda.is_available()


def gpu_partial(q, k, v, qp, kp, **kw):
    o, l = B.cp_attn_partial(dev(q), dev(k), dev(v), i32(qp), i32(kp), **kw)
    torch.cuda.synchronize()
    return o, l


# ---------------------------------------------------------------------------
# tiny pass-KV ring (fp32, d=64, GQA 4:1, 2 virtual ranks over 4 chunks of 128)
# ---------------------------------------------------------------------------

def test_tiny_passkv_ring_fp32(oracle):
    w = W.WORKLOADS["tiny_passkv"]
    q, k, v = W.qkv(w)
    q64, k64, v64 = W.to_f64(q), W.to_f64(k), W.to_f64(v)
    n = w.n_ranks
    pos = [B.cp_shard_positions(w.t_new, n, r) for r in range(n)]
    np.testing.assert_array_equal(pos[0], np.r_[0:128, 384:512])
    ref_o, ref_l = oracle.unsharded_causal(q64, k64, v64)
    o_o, o_l, po, pl = oracle.ring_passkv([q64[p] for p in pos], [k64[p] for p in pos],
                                          [v64[p] for p in pos], pos, pos)
    ring = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                  [i32(p) for p in pos], [i32(p) for p in pos], keep_partials=True)
    out, lse = B.cp_ring_passkv(ring)
    torch.cuda.synchronize()
    for a in range(n):
        for b in range(n):
            check(*ring.partial(a, b), po[a][b], pl[a][b], O_ATOL_FP32, LSE_RTOL_FP32,
                  "partial %d,%d" % (a, b))
        check(out[a], lse[a], ref_o[pos[a]], ref_l[pos[a]], O_ATOL_FP32, LSE_RTOL_FP32,
              "merged rank %d" % a)
        np.testing.assert_allclose(o_o[a], ref_o[pos[a]], atol=1e-12)


@pytest.mark.parametrize("dtype,d,nh,nkv", [("fp32", 128, 2, 2), ("bf16", 64, 8, 2),
                                            ("fp32", 64, 3, 1)])
def test_vector_kernel_shapes(oracle, dtype, d, nh, nkv):
    tq, tkv = 37, 203
    q, q64 = randn(1, (tq, nh, d), dtype)
    k, k64 = randn(2, (tkv, nkv, d), dtype)
    v, v64 = randn(3, (tkv, nkv, d), dtype)
    rng = np.random.default_rng(4)
    qp = rng.integers(-1, 260, size=tq)
    kp = rng.permutation(300)[:tkv]
    ref = oracle.attn(q64, k64, v64, qp, kp)
    o, l = gpu_partial(q, k, v, qp, kp, out_dtype=torch.float32)
    if dtype == "fp32":
        check(o, l, *ref, O_ATOL_FP32, LSE_RTOL_FP32)
    else:
        check(o, l, *ref)


def test_vector_kernel_packed_batch(oracle):
    cu_q = np.array([0, 5, 5, 40, 41], dtype=np.int32)
    cu_kv = np.array([0, 70, 90, 90, 300], dtype=np.int32)
    q, q64 = randn(5, (41, 4, 64), "fp32")
    k, k64 = randn(6, (300, 2, 64), "fp32")
    v, v64 = randn(7, (300, 2, 64), "fp32")
    rng = np.random.default_rng(8)
    qp, kp = rng.integers(0, 200, size=41), rng.integers(0, 200, size=300)
    ref = oracle.attn(q64, k64, v64, qp, kp, cu_q=cu_q, cu_kv=cu_kv)
    o, l = gpu_partial(q, k, v, qp, kp, cu_seqlens_q=i32(cu_q), cu_seqlens_kv=i32(cu_kv))
    check(o, l, *ref, O_ATOL_FP32, LSE_RTOL_FP32)


# ---------------------------------------------------------------------------
# bf16 MFMA kernel, head_dim 128
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("tq,tkv,nh,nkv", [
    (300, 777, 16, 1),    # ragged row block (4800 rows) and ragged KV tile (777 = 12*64 + 9)
    (16, 64, 16, 1),      # exactly one row block, one tile
    (1, 1, 16, 1),
    (65, 130, 8, 2),      # two KV heads, group of 4
    (40, 500, 4, 4),      # MHA: group of 1
    (33, 257, 24, 1),     # group of 24 (rows of one token straddle wavefronts)
])
def test_mfma_partial_random_positions(oracle, tq, tkv, nh, nkv):
    q, q64 = randn(11, (tq, nh, 128))
    k, k64 = randn(12, (tkv, nkv, 128))
    v, v64 = randn(13, (tkv, nkv, 128))
    rng = np.random.default_rng(14)
    qp = rng.integers(-1, tkv + 40, size=tq)
    kp = rng.permutation(tkv + 50)[:tkv]
    if tkv > 8:
        kp[rng.integers(0, tkv, size=5)] = B.CP_POS_PAD_KV   # padded slots
    ref = oracle.attn(q64, k64, v64, qp, kp)
    for odt in (torch.float32, torch.bfloat16):
        o, l = gpu_partial(q, k, v, qp, kp, out_dtype=odt)
        check(o, l, *ref, what="out dtype %s" % odt)


def test_mfma_partial_padded_queries_among_fully_visible_tiles(oracle):
    """Padded query tokens (CP_POS_PAD_Q) inside wavefronts whose other rows see every key: the
    wavefront keeps the mask-free softmax form, the padded rows still come out as O = 0,
    LSE = -inf. Unsplit walk (128 row blocks) and a split one."""
    for tq, tkv in ((2048, 1100), (160, 1100)):
        q, q64 = randn(71, (tq, 16, 128))
        k, k64 = randn(72, (tkv, 1, 128))
        v, v64 = randn(73, (tkv, 1, 128))
        kp = np.arange(tkv)
        qp = np.arange(tq) + tkv               # every key visible to every real query
        qp[[0, 3, 17, 64, 65, tq // 2, tq - 1]] = B.CP_POS_PAD_Q
        ref = oracle.attn(q64, k64, v64, qp, kp)
        assert np.isneginf(ref[1][3]).all() and np.isfinite(ref[1][4]).all()
        for odt in (torch.float32, torch.bfloat16):
            o, l = gpu_partial(q, k, v, qp, kp, out_dtype=odt)
            check(o, l, *ref, what="padded queries, tq %d, out %s" % (tq, odt))


def test_mfma_partial_seeded_shape_sweep(oracle):
    """Twelve seeded shapes inside the documented limits: ragged row blocks and tiles, every
    head grouping, split and unsplit walks, sorted and shuffled positions, pads."""
    rng = np.random.default_rng(2024)
    for case in range(12):
        nkv = int(rng.choice([1, 1, 2, 4]))
        group = int(rng.choice([1, 2, 4, 8, 16]))
        nh = nkv * group
        tq = int(rng.integers(1, 700)) if case % 3 else int(rng.integers(2048, 2600))
        tkv = int(rng.integers(1, 1500))
        q, q64 = randn(900 + case, (tq, nh, 128))
        k, k64 = randn(930 + case, (tkv, nkv, 128))
        v, v64 = randn(960 + case, (tkv, nkv, 128))
        if case % 2:
            kp = np.sort(rng.choice(3 * tkv, size=tkv, replace=False))     # a sorted shard
            qp = np.sort(rng.integers(0, 3 * tkv, size=tq))
        else:
            kp = rng.permutation(tkv + 50)[:tkv]
            qp = rng.integers(-1, tkv + 40, size=tq)
        if tkv > 8:
            kp[rng.integers(0, tkv, size=3)] = B.CP_POS_PAD_KV
        ref = oracle.attn(q64, k64, v64, qp, kp)
        o, l = gpu_partial(q, k, v, qp, kp, out_dtype=torch.float32)
        check(o, l, *ref, what="case %d: tq %d tkv %d heads %d/%d" % (case, tq, tkv, nh, nkv))


@pytest.mark.parametrize("nh,nkv", [(16, 1), (8, 2)])
def test_mfma_packed_batch_random_positions(oracle, nh, nkv):
    # Algorithm 2's fused variable-length inputs: several sequences in one call, one of them
    # empty on both sides, one with queries but no keys; random (unsorted) positions whose
    # ranges overlap between sequences, padded slots on both sides
    cu_q = np.array([0, 37, 37, 300, 310, 700], dtype=np.int32)
    cu_kv = np.array([0, 500, 500, 1300, 1300, 2100], dtype=np.int32)
    tq, tkv = int(cu_q[-1]), int(cu_kv[-1])
    q, q64 = randn(41, (tq, nh, 128))
    k, k64 = randn(42, (tkv, nkv, 128))
    v, v64 = randn(43, (tkv, nkv, 128))
    rng = np.random.default_rng(44)
    qp = rng.integers(-1, 900, size=tq)
    kp = rng.integers(0, 900, size=tkv)
    kp[rng.integers(0, tkv, size=9)] = B.CP_POS_PAD_KV
    ref = oracle.attn(q64, k64, v64, qp, kp, cu_q=cu_q, cu_kv=cu_kv)
    assert np.isneginf(ref[1][300:310]).all()       # the sequence without keys
    for odt in (torch.float32, torch.bfloat16):
        o, l = gpu_partial(q, k, v, qp, kp, cu_seqlens_q=i32(cu_q), cu_seqlens_kv=i32(cu_kv),
                           out_dtype=odt)
        check(o, l, *ref, what="packed batch, out dtype %s" % odt)


def test_mfma_packed_batch_causal_prefill_with_cache_offsets(oracle):
    # three sequences of different length, each a partial prefill: cached positions 0..P_b-1
    # plus T_b new tokens at P_b..P_b+T_b-1; sorted positions, so every tile class occurs
    # (skipped, unmasked, straddling a sequence boundary, straddling the diagonal)
    p_cached = [0, 900, 130]
    t_new = [700, 150, 260]
    cu_q = np.concatenate([[0], np.cumsum(t_new)]).astype(np.int32)
    cu_kv = np.concatenate([[0], np.cumsum([p + t for p, t in zip(p_cached, t_new)])]).astype(np.int32)
    qp = np.concatenate([np.arange(p, p + t) for p, t in zip(p_cached, t_new)])
    kp = np.concatenate([np.arange(0, p + t) for p, t in zip(p_cached, t_new)])
    tq, tkv = int(cu_q[-1]), int(cu_kv[-1])
    q, q64 = randn(51, (tq, 16, 128))
    k, k64 = randn(52, (tkv, 1, 128))
    v, v64 = randn(53, (tkv, 1, 128))
    ref = oracle.attn(q64, k64, v64, qp, kp, cu_q=cu_q, cu_kv=cu_kv)
    o, l = gpu_partial(q, k, v, qp, kp, cu_seqlens_q=i32(cu_q), cu_seqlens_kv=i32(cu_kv),
                       out_dtype=torch.float32)
    check(o, l, *ref, what="packed causal prefill")
    # the same rows through one call per sequence (batch 1) must agree with the oracle too
    for b in range(3):
        qs, ks = slice(cu_q[b], cu_q[b + 1]), slice(cu_kv[b], cu_kv[b + 1])
        o1, l1 = gpu_partial(q[qs], k[ks], v[ks], qp[qs], kp[ks], out_dtype=torch.float32)
        check(o1, l1, ref[0][qs], ref[1][qs], what="sequence %d alone" % b)


def test_mfma_partial_sorted_positions_all_tile_classes(oracle):
    # natural causal order: tiles are skipped, unmasked, or diagonal depending on the row block
    t = 700
    q, q64 = randn(21, (t, 16, 128))
    k, k64 = randn(22, (t, 1, 128))
    v, v64 = randn(23, (t, 1, 128))
    pos = np.arange(t)
    ref = oracle.attn(q64, k64, v64, pos, pos)
    o, l = gpu_partial(q, k, v, pos, pos, out_dtype=torch.float32)
    check(o, l, *ref)


def test_mfma_partial_softmax_scale_and_short_rows(oracle):
    # explicit scale; row 0 sees one key (LSE ~ N(0,1), O = v0 exactly up to bf16 products)
    t = 130
    q, q64 = randn(31, (t, 16, 128))
    k, k64 = randn(32, (t, 1, 128))
    v, v64 = randn(33, (t, 1, 128))
    pos = np.arange(t)
    ref = oracle.attn(q64, k64, v64, pos, pos, scale=0.05)
    o, l = gpu_partial(q, k, v, pos, pos, out_dtype=torch.float32, softmax_scale=0.05)
    check(o, l, *ref)
    np.testing.assert_allclose(o[0].cpu().double().numpy(), np.broadcast_to(v64[0], (16, 128)),
                               atol=1e-6)


@pytest.mark.parametrize("causal,tq", [(False, 96), (True, 96), (False, 2048)])
def test_mfma_partial_score_spikes(oracle, causal, tq):
    # Keys whose score lies far above everything seen before them (45 and then 80 log2 units
    # above the running reference), and one far below: the kernel's softmax keeps a standing
    # reference without looking at block maxima and must notice such blocks and redo them.
    # The spikes sit in the second and third 32-key block of their 128-key tile, so a
    # reference exists when they arrive, also where the KV axis is split per tile (tq = 96);
    # tq = 2048 is the unsplit walk over all tiles.
    t = 600
    u, _ = randn(41, (128,))
    noise, _ = randn(42, (tq, 16, 128))
    q = (u.float()[None, None, :] + 0.1 * noise.float()).to(torch.bfloat16)
    k, _ = randn(43, (t, 1, 128))
    v, v64 = randn(44, (t, 1, 128))
    k = k.clone()
    k[182, 0] = (3.0 * u.float()).to(torch.bfloat16)
    k[183, 0] = (-6.0 * u.float()).to(torch.bfloat16)
    k[464, 0] = (5.0 * u.float()).to(torch.bfloat16)
    q64, k64 = W.to_f64(q), W.to_f64(k)
    kp = np.arange(t)
    qp = np.linspace(5, t - 1, tq).astype(np.int64) if causal else np.full(tq, 10**6)
    ref = oracle.attn(q64, k64, v64, qp, kp)
    o, l = gpu_partial(q, k, v, qp, kp, out_dtype=torch.float32)
    check(o, l, *ref)
    sees_big = qp >= 464
    assert sees_big.any()
    # rows that see the largest spike are that key's value row, to bf16 rounding of P
    np.testing.assert_allclose(o[sees_big].cpu().double().numpy(),
                               np.broadcast_to(v64[464], (int(sees_big.sum()), 16, 128)), atol=1e-2)


def test_ring_fused_merge_matches_unsharded(oracle):
    # the drivers' fused-merge option (running result in the epilogues, no partials, no merge
    # pass) in both ring orders; t = 16384 keeps every call unsplit, which the option needs
    n, t = 2, 16384
    q, q64 = randn(41, (t, 16, 128))
    k, k64 = randn(42, (t, 1, 128))
    v, v64 = randn(43, (t, 1, 128))
    pos = [B.cp_shard_positions(t, n, r) for r in range(n)]
    rows = np.r_[0:64, 4090:4102, 8190:8200, 12280:12296, t - 64:t]  # oracle on a sample of rows
    ref_o, ref_l = oracle.attn(q64[rows], k64, v64, rows, np.arange(t))
    where = {int(p): (a, i) for a in range(n) for i, p in enumerate(pos[a])}
    for order in (B.cp_ring_passkv, B.cp_ring_passq):
        ring = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                      [i32(p) for p in pos], [i32(p) for p in pos], out_dtype=torch.float32,
                      fused_merge=True)
        assert ring.partial_out.shape[0] == 1
        out, lse = order(ring)
        torch.cuda.synchronize()
        got_o = torch.stack([out[where[int(r)][0]][where[int(r)][1]] for r in rows])
        got_l = torch.stack([lse[where[int(r)][0]][where[int(r)][1]] for r in rows])
        check(got_o, got_l, ref_o, ref_l, what=order.__name__)
    small = B.Ring([dev(q[p][:64]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                   [i32(p[:64]) for p in pos], [i32(p) for p in pos], fused_merge=True)
    with pytest.raises(B.CpError):  # short query shards split the KV axis: not supported
        B.cp_ring_passkv(small)


@pytest.mark.parametrize("n,t,flags", [(4, 8192, False), (4, 8192, True), (3, 6144 + 3 * 256, False),
                                       (3, 7001, True)])
def test_ring_walk_in_one_launch_matches_unsharded(oracle, n, t, flags):
    """fused_merge=2: every rank's N ring steps in one launch, with and without arrival
    flags (all set before the call), fp32 and bf16 outputs, with and without the LSE."""
    q, q64 = randn(51, (t, 16, 128))
    k, k64 = randn(52, (t, 1, 128))
    v, v64 = randn(53, (t, 1, 128))
    pos = [B.cp_shard_positions(t, n, r) for r in range(n)]
    # (t = 7001: shards of 2334, 2334 and 2333 tokens, ragged last tiles)
    rows = np.r_[0:48, t // 4 - 6:t // 4 + 6, t // 2 - 5:t // 2 + 5, t - 3 * t // 8:t - 3 * t // 8 + 16,
                 t - 48:t]
    # one padded query row (sees nothing in any shard): token 5, the sixth row of rank 0
    rows = rows[rows != 5]
    q_pos = [p.copy() for p in pos]
    assert pos[0][5] == 5
    q_pos[0][5] = B.CP_POS_PAD_Q
    ref_o, ref_l = oracle.attn(q64[rows], k64, v64, rows, np.arange(t))
    where = {int(p): (a, i) for a in range(n) for i, p in enumerate(pos[a])}
    for odt in (torch.float32, torch.bfloat16):
        arrived = [torch.ones(n, dtype=torch.int32, device="cuda") for _ in range(n)] \
            if flags else None
        ring = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                      [i32(p) for p in q_pos], [i32(p) for p in pos], out_dtype=odt,
                      fused_merge=2, arrived=arrived, spin_limit=1000)
        out, lse = B.cp_ring_passkv(ring)
        torch.cuda.synchronize()
        if flags:
            assert not ring.arrival_failed()
        assert torch.isneginf(lse[0][5]).all() and (out[0][5] == 0).all()
        got_o = torch.stack([out[where[int(r)][0]][where[int(r)][1]] for r in rows])
        got_l = torch.stack([lse[where[int(r)][0]][where[int(r)][1]] for r in rows])
        check(got_o, got_l, ref_o, ref_l, what="ring walk, %s" % odt)
        # the step-by-step ring with the merge in the epilogues computes the same thing
        if odt == torch.float32:
            step = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos],
                          [dev(v[p]) for p in pos], [i32(p) for p in q_pos], [i32(p) for p in pos],
                          out_dtype=odt, fused_merge=True)
            out_s, lse_s = B.cp_ring_passkv(step)
            torch.cuda.synchronize()
            for a in range(n):
                assert float((out[a] - out_s[a]).abs().max()) < 2e-3
                fin = torch.isfinite(lse[a])
                assert torch.equal(fin, torch.isfinite(lse_s[a]))
                assert float((lse[a][fin] - lse_s[a][fin]).abs().max()) < 1e-4
    with pytest.raises(B.CpError):   # pass-Q moves the queries: no such walk
        B.cp_ring_passq(ring)


@pytest.mark.parametrize("fused", [0, 1, 2])
def test_ring_with_an_empty_and_uneven_kv_shards(oracle, fused):
    """The KV of a ring need not be sharded like the queries (the mask is by position): one
    rank holds no keys at all, another two ranks' worth, the third a ragged count. Covers the
    one-launch tile-bound pre-pass over shards of different sizes, an empty one among them."""
    n, t = 3, 6144 + 77
    q, q64 = randn(61, (t, 16, 128))
    k, k64 = randn(62, (t, 1, 128))
    v, v64 = randn(63, (t, 1, 128))
    pos = [B.cp_shard_positions(t, n, r) for r in range(n)]
    kv = [np.concatenate([pos[0], pos[1][:-5]]), np.zeros(0, dtype=np.int32),
          np.concatenate([pos[2], pos[1][-5:]])]
    rows = np.r_[0:40, t // 2 - 8:t // 2 + 8, t - 40:t]
    ref_o, ref_l = oracle.attn(q64[rows], k64, v64, rows, np.arange(t))
    where = {int(p): (a, i) for a in range(n) for i, p in enumerate(pos[a])}
    ring = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in kv], [dev(v[p]) for p in kv],
                  [i32(p) for p in pos], [i32(p) for p in kv], out_dtype=torch.float32,
                  fused_merge=fused)
    out, lse = B.cp_ring_passkv(ring)
    torch.cuda.synchronize()
    got_o = torch.stack([out[where[int(r)][0]][where[int(r)][1]] for r in rows])
    got_l = torch.stack([lse[where[int(r)][0]][where[int(r)][1]] for r in rows])
    check(got_o, got_l, ref_o, ref_l, what="ring with an empty KV shard, fused_merge=%d" % fused)


def test_ring_walk_gives_up_on_a_shard_that_never_arrives(oracle):
    """The host never sets one step's flag and allows three polls: every kernel still ends,
    the error word is set, and the ranks whose flags were all set are unaffected."""
    n, t = 4, 8192
    q, q64 = randn(51, (t, 16, 128))
    k, k64 = randn(52, (t, 1, 128))
    v, v64 = randn(53, (t, 1, 128))
    pos = [B.cp_shard_positions(t, n, r) for r in range(n)]
    arrived = [torch.ones(n, dtype=torch.int32, device="cuda") for _ in range(n)]
    arrived[2][1] = 0          # rank 2 never receives the shard of its step 1
    ring = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                  [i32(p) for p in pos], [i32(p) for p in pos], out_dtype=torch.float32,
                  fused_merge=2, arrived=arrived, spin_limit=3)
    out, lse = B.cp_ring_passkv(ring)
    torch.cuda.synchronize()
    # rank 2, step 1 and nothing else
    assert ring.ring_error.tolist() == [0, 0, 1 << 1, 0] and ring.arrival_failed()
    rows = np.r_[0:16, 1000:1016, 2032:2048]
    for a in (0, 1, 3):
        tok = pos[a][rows]
        ref_o, ref_l = oracle.attn(q64[tok], k64, v64, tok, np.arange(t))
        check(out[a][rows], lse[a][rows], ref_o, ref_l, what="rank %d" % a)
    # rank 2 computed attention over everything but the missing shard (KV of rank 1)
    keep = np.concatenate([pos[s] for s in (0, 2, 3)])
    tok = pos[2][rows]
    ref_o, ref_l = oracle.attn(q64[tok], k64[keep], v64[keep], tok, keep)
    check(out[2][rows], lse[2][rows], ref_o, ref_l, what="rank 2 without the shard of rank 1")


@pytest.mark.parametrize("n,t,two_streams", [(4, 2048, False), (3, 1000, False),
                                             (4, 2048, True), (2, 16384, True)])
def test_mfma_load_balanced_partials_and_merge(oracle, n, t, two_streams):
    # two_streams: the drivers issue a rank's calls alternately on two streams (t = 16384 gives
    # every call enough row blocks that none splits its KV axis, the condition for doing so)
    aux = torch.cuda.Stream() if two_streams else None
    q, q64 = randn(41, (t, 16, 128))
    k, k64 = randn(42, (t, 1, 128))
    v, v64 = randn(43, (t, 1, 128))
    pos = [B.cp_shard_positions(t, n, r) for r in range(n)]
    ref_o, ref_l = oracle.unsharded_causal(q64, k64, v64)
    ring = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                  [i32(p) for p in pos], [i32(p) for p in pos], keep_partials=True,
                  out_dtype=torch.float32, aux_stream=aux)
    out, lse = B.cp_ring_passkv(ring)
    torch.cuda.synchronize()
    for a in range(n):
        for b in range(n):
            if t > 4096 and (a, b) != (n - 1, 0):
                continue  # the oracle's time: one partial of the large case is enough
            po, pl = oracle.attn(q64[pos[a]], k64[pos[b]], v64[pos[b]], pos[a], pos[b])
            check(*ring.partial(a, b), po, pl, what="partial %d,%d" % (a, b))
        check(out[a], lse[a], ref_o[pos[a]], ref_l[pos[a]], what="merged rank %d" % a)
    # pass-Q order over the same shards gives the same merged result
    ring_q = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                    [i32(p) for p in pos], [i32(p) for p in pos], out_dtype=torch.float32,
                    aux_stream=aux)
    out_q, lse_q = B.cp_ring_passq(ring_q)
    torch.cuda.synchronize()
    for a in range(n):
        check(out_q[a], lse_q[a], ref_o[pos[a]], ref_l[pos[a]], what="pass-Q rank %d" % a)


def test_ring_passkv_bf16_partials(oracle):
    # partial outputs stored as bf16 (LSE stays fp32): merged result within the same bar
    n, t = 4, 2048
    q, q64 = randn(45, (t, 16, 128))
    k, k64 = randn(46, (t, 1, 128))
    v, v64 = randn(47, (t, 1, 128))
    pos = [B.cp_shard_positions(t, n, r) for r in range(n)]
    ref_o, ref_l = oracle.unsharded_causal(q64, k64, v64)
    ring = B.Ring([dev(q[p]) for p in pos], [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                  [i32(p) for p in pos], [i32(p) for p in pos], keep_partials=True,
                  out_dtype=torch.bfloat16, part_dtype=torch.bfloat16)
    out, lse = B.cp_ring_passkv(ring)
    torch.cuda.synchronize()
    for a in range(n):
        check(out[a], lse[a], ref_o[pos[a]], ref_l[pos[a]], what="merged rank %d" % a)
    po, pl = oracle.attn(q64[pos[3]], k64[pos[1]], v64[pos[1]], pos[3], pos[1])
    check(*ring.partial(3, 1), po, pl, what="bf16 partial 3,1")


@pytest.mark.parametrize("final_dtype", [torch.float32, torch.bfloat16])
def test_partial_accumulate_matches_attention_on_the_union(oracle, final_dtype):
    # three steps merged in the kernel's epilogue == attention over the three KV sets together
    tq, nkv = 2048, 3
    q, q64 = randn(61, (tq, 16, 128))
    rng = np.random.default_rng(62)
    qp = rng.integers(0, 1500, size=tq)
    qp[:5] = -1            # padded queries: see nothing in any step
    qp[5:40] = 700         # see all of step 0, part of step 1, nothing of step 2
    ks, vs, kps = [], [], []
    for i in range(nkv):
        n_k = (300, 421, 256)[i]
        k, _ = randn(63 + i, (n_k, 1, 128))
        v, _ = randn(73 + i, (n_k, 1, 128))
        ks.append(k); vs.append(v)
        kps.append(rng.permutation(500)[:n_k] + 500 * i)
    acc_o = torch.empty((tq, 16, 128), dtype=torch.float32, device="cuda")
    acc_l = torch.empty((tq, 16), dtype=torch.float32, device="cuda")
    fin_o = torch.empty((tq, 16, 128), dtype=final_dtype, device="cuda")
    fin_l = torch.empty((tq, 16), dtype=torch.float32, device="cuda")
    dq, dqp = dev(q), i32(qp)
    B.cp_attn_partial(dq, dev(ks[0]), dev(vs[0]), dqp, i32(kps[0]), out=acc_o, lse=acc_l)
    B.cp_attn_partial_accumulate(dq, dev(ks[1]), dev(vs[1]), dqp, i32(kps[1]), acc_o, acc_l)
    torch.cuda.synchronize()
    ref2 = oracle.attn(q64, np.concatenate([W.to_f64(x) for x in ks[:2]]),
                       np.concatenate([W.to_f64(x) for x in vs[:2]]), qp, np.concatenate(kps[:2]))
    check(acc_o, acc_l, *ref2, what="running result after two steps")
    before = acc_o.clone()
    B.cp_attn_partial_accumulate(dq, dev(ks[2]), dev(vs[2]), dqp, i32(kps[2]), acc_o, acc_l,
                                 final_out=fin_o, final_lse=fin_l)
    torch.cuda.synchronize()
    ref3 = oracle.attn(q64, np.concatenate([W.to_f64(x) for x in ks]),
                       np.concatenate([W.to_f64(x) for x in vs]), qp, np.concatenate(kps))
    check(fin_o, fin_l, *ref3, what="final output")
    check(fin_o, acc_l, *ref3, what="running LSE after the last step")
    assert torch.equal(acc_o, before)  # the last step writes the final output only
    assert np.isneginf(ref3[1][:5]).all() and not np.isneginf(ref3[1][5:]).any()


def test_mfma_split_kv_short_query_shard(oracle):
    # 40 query tokens x 16 heads (3 row blocks) against 3000 keys: the KV axis is split
    tq, tkv = 40, 3000
    shape = B.make_shape(B.CP_BF16, 128, 16, 1, tq, tkv)
    assert B.cp_workspace_bytes(shape, B.CP_WS_PARTIAL) > tq * 16 * 128 * 4 * 2
    q, q64 = randn(51, (tq, 16, 128))
    k, k64 = randn(52, (tkv, 1, 128))
    v, v64 = randn(53, (tkv, 1, 128))
    qp = np.arange(tkv - tq, tkv)
    qp[3] = B.CP_POS_PAD_Q
    kp = np.arange(tkv)
    ref = oracle.attn(q64, k64, v64, qp, kp)
    for odt in (torch.float32, torch.bfloat16):
        o, l = gpu_partial(q, k, v, qp, kp, out_dtype=odt)
        check(o, l, *ref)


def test_partial_degenerate_inputs(oracle):
    q, q64 = randn(61, (20, 16, 128))
    k, k64 = randn(62, (100, 1, 128))
    v, v64 = randn(63, (100, 1, 128))
    # no keys at all
    o, l = B.cp_attn_partial(dev(q), dev(k[:0]), dev(v[:0]), i32(np.arange(20)), i32([]),
                             out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.all(o == 0) and torch.all(torch.isneginf(l))
    # every key beyond every query
    o, l = gpu_partial(q, k, v, np.arange(20), np.arange(100) + 1000, out_dtype=torch.float32)
    assert torch.all(o == 0) and torch.all(torch.isneginf(l))
    # no queries
    o, l = B.cp_attn_partial(dev(q[:0]), dev(k), dev(v), i32([]), i32(np.arange(100)))
    assert o.shape == (0, 16, 128)


# ---------------------------------------------------------------------------
# merge (Equation 4)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n_parts", [1, 2, 3, 16, 17])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_merge_matches_oracle(oracle, n_parts, pdt):
    rows, d = (37, 16), 128
    rng = np.random.default_rng(70 + n_parts)
    outs = [torch.from_numpy(rng.standard_normal(rows + (d,))).to(pdt) for _ in range(n_parts)]
    lses = [rng.standard_normal(rows) * 4 for _ in range(n_parts)]
    for s in range(n_parts):
        lses[s][rng.integers(0, rows[0], 6), rng.integers(0, rows[1], 6)] = -np.inf
    for s in range(n_parts):
        lses[s][5, :] = -np.inf                       # a row that is empty in every partial
        outs[s][lses_mask(lses[s])] = float("nan")    # O of an empty partial must not be read
    ref_o, ref_l = oracle.merge([W.to_f64(o) for o in outs], lses)
    for odt in (torch.float32, torch.bfloat16):
        o, l = B.cp_attn_merge([dev(x) for x in outs], [dev(x, torch.float32) for x in lses],
                               out_dtype=odt)
        torch.cuda.synchronize()
        check(o, l, ref_o, ref_l, o_atol=1e-5 if odt == torch.float32 else 2e-2,
              lse_rtol=1e-5)


def lses_mask(l):
    return torch.from_numpy(np.isneginf(l))


def test_merge_large_stream(oracle):
    # enough rows for the grid-stride loop to wrap (more than 8192 workgroups of 256 slices)
    rows, d, n = 70001, 128, 4
    rng = np.random.default_rng(81)
    outs = [torch.from_numpy(rng.standard_normal((rows, d)).astype(np.float32)) for _ in range(n)]
    lses = [rng.standard_normal(rows).astype(np.float32) for _ in range(n)]
    ref_o, ref_l = oracle.merge([x.numpy() for x in outs], lses)
    o, l = B.cp_attn_merge([dev(x) for x in outs], [dev(x) for x in lses])
    torch.cuda.synchronize()
    check(o, l, ref_o, ref_l, o_atol=1e-5, lse_rtol=1e-5)


# ---------------------------------------------------------------------------
# split-KV decode (Algorithm 4)
# ---------------------------------------------------------------------------

def _decode_case(oracle, lengths, nh, nkv, bid, seed, pad_some=False, unique_bid=False):
    total = int(np.sum(lengths))
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    nq = len(bid)
    q, q64 = randn(seed, (nq, nh, 128))
    k, k64 = randn(seed + 1, (total, nkv, 128))
    v, v64 = randn(seed + 2, (total, nkv, 128))
    kp = np.concatenate([np.arange(n) for n in lengths]).astype(np.int32)
    qp = np.array([max(lengths[b] - 1, 0) for b in bid], dtype=np.int32)
    if pad_some:
        rng = np.random.default_rng(seed)
        kp[rng.integers(0, total, size=7)] = B.CP_POS_PAD_KV
        qp[0] = lengths[bid[0]] // 2          # a query that sees only half of its segment
    segs = [np.arange(cu[b], cu[b + 1]) for b in bid]
    idx = np.concatenate(segs)
    cu_sel = np.concatenate([[0], np.cumsum([len(s) for s in segs])]).astype(np.int32)
    ref = oracle.attn(q64, k64[idx], v64[idx], qp, kp[idx],
                      cu_q=np.arange(nq + 1, dtype=np.int32), cu_kv=cu_sel)
    for odt in (torch.float32, torch.bfloat16):
        o, l = B.cp_attn_decode(dev(q), dev(k), dev(v), i32(qp), i32(kp), i32(cu), i32(bid),
                                out_dtype=odt, unique_bid=unique_bid)
        torch.cuda.synchronize()
        check(o, l, *ref, what="decode out %s%s" % (odt, " (flat ranges)" if unique_bid else ""))


def test_decode_varied_lengths(oracle):
    _decode_case(oracle, [1000, 1, 33, 4097, 0, 260, 129], 16, 1, [0, 1, 2, 3, 4, 5, 6], 90)


def test_decode_subset_of_sequences_permuted(oracle):
    _decode_case(oracle, [500, 900, 64, 2000, 31], 16, 1, [3, 0, 3, 4], 93, pad_some=True)


def test_decode_smaller_groups(oracle):
    _decode_case(oracle, [300, 700, 1500], 8, 2, [2, 0, 1], 96)
    _decode_case(oracle, [300, 700], 4, 4, [1, 0], 99)


# The flat path (CP_SHAPE_UNIQUE_BID): equal key ranges per workgroup regardless of the sequence
# boundaries. The cases put boundaries inside ranges and inside tiles, leave sequences without
# a query, and include empty and one-key sequences.
@pytest.mark.parametrize("lengths,bid", [
    ([1000, 1, 33, 4097, 0, 260, 129], [0, 1, 2, 3, 4, 5, 6]),
    ([500, 900, 64, 2000, 31], [3, 0, 4]),                 # permuted, two sequences unasked
    ([7, 3, 1, 0, 0, 2, 40, 5, 9, 1], [9, 8, 7, 6, 5, 4, 3, 2, 1, 0]),   # many ends in one tile
    ([8192 * 3 + 17, 5000, 12345], [2, 1, 0]),             # several tiles per wavefront
    ([32 * 256], [0]),                                     # ranges end exactly on the sequence
    ([64] * 64, list(range(63, -1, -1))),                  # a boundary at every range end
])
def test_decode_flat_ranges(oracle, lengths, bid):
    _decode_case(oracle, lengths, 16, 1, bid, 120 + len(lengths), unique_bid=True)


def test_decode_flat_more_sequences_than_table_lanes(oracle):
    """More than 64 sequences and queries: the entries of cu_seqlens_kv, bid and q_pos past the
    per-lane tables come through scalar loads, the first sequence of a range by bisection."""
    rng = np.random.default_rng(77)
    lengths = [int(x) for x in rng.integers(0, 400, size=150)]
    bid = [int(x) for x in rng.permutation(150)]
    _decode_case(oracle, lengths, 16, 1, bid, 141, unique_bid=True)
    # queries for the late sequences only: every lookup misses the 64-entry bid table first
    _decode_case(oracle, lengths, 16, 1, list(range(149, 69, -1)), 142, unique_bid=True)


def test_decode_flat_ranges_pads_and_groups(oracle):
    _decode_case(oracle, [500, 900, 64, 2000, 31], 16, 1, [3, 0, 1, 4], 131, pad_some=True,
                 unique_bid=True)
    _decode_case(oracle, [300, 700, 1500], 8, 2, [2, 0, 1], 134, unique_bid=True)
    _decode_case(oracle, [300, 700], 4, 4, [1, 0], 137, unique_bid=True)


def test_ring_passq_decode_driver(oracle):
    n, nh = 4, 16
    lengths = [900, 35, 2300, 1, 640, 1200, 77, 3000]
    rng = np.random.default_rng(101)
    ks = [W.normal(200 + b, (L, 1, 128)) for b, L in enumerate(lengths)]
    vs = [W.normal(300 + b, (L, 1, 128)) for b, L in enumerate(lengths)]
    qs = [W.normal(400 + b, (1, nh, 128)) for b in range(len(lengths))]
    ranks = oracle.shard_decode_batch(lengths, n, decode_iter=1)

    def gather(src, r):
        if len(r["kv_pos"]) == 0:
            return torch.zeros((0, 1, 128), dtype=torch.bfloat16)
        return torch.cat([src[b][p][None] for b, p in zip(r["kv_seq"], r["kv_pos"])])
    rk = [gather(ks, r) for r in ranks]
    rv = [gather(vs, r) for r in ranks]
    rq = [torch.cat([qs[b] for b in r["bid"]]) if len(r["bid"]) else
          torch.zeros((0, nh, 128), dtype=torch.bfloat16) for r in ranks]
    ref_o, ref_l, _, _ = oracle.ring_passq_decode(
        [W.to_f64(x) for x in rq], [r["bid"] for r in ranks], [r["q_pos"] for r in ranks],
        [W.to_f64(x) for x in rk], [W.to_f64(x) for x in rv], [r["kv_pos"] for r in ranks],
        [r["cu_kv"] for r in ranks])
    for keep in (False, True):
        ring = B.Ring([dev(x) for x in rq], [dev(x) for x in rk], [dev(x) for x in rv],
                      [i32(r["q_pos"]) for r in ranks], [i32(r["kv_pos"]) for r in ranks],
                      out_dtype=torch.float32, keep_partials=keep,
                      cu_seqlens_kv=[i32(r["cu_kv"]) for r in ranks],
                      bid=[i32(r["bid"]) for r in ranks])
        out, lse = B.cp_ring_passq_decode(ring)
        torch.cuda.synchronize()
        for s in range(n):
            check(out[s], lse[s], ref_o[s], ref_l[s], what="decode ring rank %d" % s)
    # and against plain attention of every sequence on its own
    for s, r in enumerate(ranks):
        for i, b in enumerate(r["bid"]):
            L = lengths[b]
            o1, l1 = oracle.attn(W.to_f64(qs[b]), W.to_f64(ks[b]), W.to_f64(vs[b]), [L - 1],
                                 np.arange(L))
            np.testing.assert_allclose(ref_o[s][i], o1[0], atol=1e-12)


# ---------------------------------------------------------------------------
# pass-Q partial prefill driver (Algorithm 3) with a cached prefix
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("partition", ["balanced", "contiguous"])
def test_ring_passq_partial_prefill(oracle, partition):
    n, p_cached, t_new = 4, 3000, 200
    q, q64 = randn(111, (t_new, 16, 128))
    k, k64 = randn(112, (p_cached + t_new, 1, 128))
    v, v64 = randn(113, (p_cached + t_new, 1, 128))
    ref_o, ref_l = oracle.unsharded_causal(q64, k64, v64, p_cached=p_cached)
    sh = oracle.shard_partial_prefill(p_cached, t_new, n, cache_partition=partition)
    ring = B.Ring([dev(q[qp - p_cached]) for qp, _ in sh], [dev(k[kp]) for _, kp in sh],
                  [dev(v[kp]) for _, kp in sh], [i32(qp) for qp, _ in sh],
                  [i32(kp) for _, kp in sh], out_dtype=torch.float32)
    out, lse = B.cp_ring_passq(ring)
    torch.cuda.synchronize()
    for r, (qp, _) in enumerate(sh):
        check(out[r], lse[r], ref_o[qp - p_cached], ref_l[qp - p_cached], what="rank %d" % r)
    out2, lse2 = B.cp_ring_passkv(ring)
    torch.cuda.synchronize()
    for r, (qp, _) in enumerate(sh):
        check(out2[r], lse2[r], ref_o[qp - p_cached], ref_l[qp - p_cached])


@pytest.mark.parametrize("part", ["fp32", "bf16"])
def test_ring_passq_all2all_messages(oracle, part):
    """Partials written in place as All2All messages (O of the slot, then its LSE): the raw
    buffer, decoded here from the documented layout, holds the oracle's per-(source, holder)
    partials, the N messages a rank receives are one contiguous range, and the merged
    results are those of the two-buffer layout."""
    n, p_cached, t_new, nh, d = 4, 1000, 333, 16, 128
    q, q64 = randn(121, (t_new, nh, d))
    k, k64 = randn(122, (p_cached + t_new, 1, d))
    v, v64 = randn(123, (p_cached + t_new, 1, d))
    sh = oracle.shard_partial_prefill(p_cached, t_new, n)
    qs64 = [q64[qp - p_cached] for qp, _ in sh]
    ref_o, ref_l, part_o, part_l = oracle.ring_passq(
        qs64, [k64[kp] for _, kp in sh], [v64[kp] for _, kp in sh],
        [qp for qp, _ in sh], [kp for _, kp in sh])
    pdt = torch.float32 if part == "fp32" else torch.bfloat16
    args = ([dev(q[qp - p_cached]) for qp, _ in sh], [dev(k[kp]) for _, kp in sh],
            [dev(v[kp]) for _, kp in sh], [i32(qp) for qp, _ in sh], [i32(kp) for _, kp in sh])
    ring = B.Ring(*args, out_dtype=torch.float32, part_dtype=pdt, keep_partials=True,
                  message_layout=True)
    out, lse = B.cp_ring_passq(ring)
    torch.cuda.synchronize()
    for s in range(n):
        check(out[s], lse[s], ref_o[s], ref_l[s], what="merged, source rank %d" % s)
    plain = B.Ring(*args, out_dtype=torch.float32, part_dtype=pdt, keep_partials=True)
    out_p, lse_p = B.cp_ring_passq(plain)
    torch.cuda.synchronize()
    for s in range(n):
        assert torch.equal(out[s], out_p[s]) and torch.equal(lse[s], lse_p[s])
    # the raw messages
    raw = ring.messages.cpu()
    max_q = max(len(qp) for qp, _ in sh)
    e = 4 if part == "fp32" else 2
    o_bytes, l_bytes = max_q * nh * d * e, max_q * nh * 4
    assert ring.message_bytes % 256 == 0 and 0 <= ring.message_bytes - o_bytes - l_bytes < 256
    assert raw.shape == (n * n, ring.message_bytes)
    for s in range(n):          # receiver (source of the queries)
        rows = len(sh[s][0])
        for kk in range(n):     # sender (holder of the KV): message s*n + kk
            msg = raw[s * n + kk]
            o = msg[:o_bytes].view(pdt).view(max_q, nh, d)[:rows]
            l = msg[o_bytes:o_bytes + l_bytes].view(torch.float32).view(max_q, nh)[:rows]
            check(o, l, part_o[s][kk], part_l[s][kk], what="message %d <- %d" % (s, kk))
    # without keep_partials the N reusable slots are messages too (pass-KV, pass-Q)
    small = B.Ring(*args, out_dtype=torch.float32, part_dtype=pdt, message_layout=True)
    for fn in (B.cp_ring_passq, B.cp_ring_passkv):
        o2, l2 = fn(small)
        torch.cuda.synchronize()
        for s in range(n):
            check(o2[s], l2[s], ref_o[s], ref_l[s], what="N-slot messages, rank %d" % s)


# ---------------------------------------------------------------------------
# measurement support: the streaming-read probe reads every chunk exactly once
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n_words,n_wg", [(4, 1), (4 * 256 * 8 * 3 + 52, 3), (1 << 20, 64)])
def test_hbm_read_probe_reads_every_chunk_once(n_words, n_wg):
    rng = np.random.default_rng(5)
    host = rng.integers(0, 2 ** 31 - 1, n_words, dtype=np.int32)
    buf = torch.as_tensor(host).to("cuda")
    sink = torch.zeros(n_wg * 256, dtype=torch.int32, device="cuda")
    from bench_support import probes
    assert probes.hbm_read(buf, n_wg, sink) == n_words * 4
    torch.cuda.synchronize()
    # the xor of what the threads folded is the xor of the buffer iff no chunk was skipped or
    # read twice (random words: a chunk read twice cancels, a skipped one is missing)
    assert np.bitwise_xor.reduce(sink.cpu().numpy()) == np.bitwise_xor.reduce(host)


# ---------------------------------------------------------------------------
# pass-Q with gathered queries: one call per KV holder answers all N ring steps
# ---------------------------------------------------------------------------

def test_ring_passq_gathered_queries_partial_prefill(oracle):
    n, p_cached, t_new, nh, d = 4, 3000, 256, 16, 128
    q, q64 = randn(131, (t_new, nh, d))
    k, k64 = randn(132, (p_cached + t_new, 1, d))
    v, v64 = randn(133, (p_cached + t_new, 1, d))
    sh = oracle.shard_partial_prefill(p_cached, t_new, n)
    m = len(sh[0][0])
    assert all(len(qp) == m for qp, _ in sh)
    ref_o, ref_l, part_o, part_l = oracle.ring_passq(
        [q64[qp - p_cached] for qp, _ in sh], [k64[kp] for _, kp in sh],
        [v64[kp] for _, kp in sh], [qp for qp, _ in sh], [kp for _, kp in sh])
    # the gathered buffers: shards back to back in rank order
    order = np.concatenate([qp for qp, _ in sh])
    q_all, qpos_all = dev(q[order - p_cached]), i32(order)
    qs = [q_all[s * m:(s + 1) * m] for s in range(n)]
    qps = [qpos_all[s * m:(s + 1) * m] for s in range(n)]
    kv = ([dev(k[kp]) for _, kp in sh], [dev(v[kp]) for _, kp in sh])
    ring = B.Ring(qs, kv[0], kv[1], qps, [i32(kp) for _, kp in sh], out_dtype=torch.float32,
                  keep_partials=True, gathered_q=True)
    out, lse = B.cp_ring_passq(ring)
    torch.cuda.synchronize()
    for s in range(n):
        check(out[s], lse[s], ref_o[s], ref_l[s], what="merged, source %d" % s)
        for kk in range(n):
            po, pl = ring.partial(s, kk)
            check(po, pl, part_o[s][kk], part_l[s][kk], what="partial %d vs KV %d" % (s, kk))
    # a holder's N partials are one contiguous block in destination order (its send buffer)
    assert ring.partial_out[2 * n:3 * n].is_contiguous()
    po, _ = ring.partial(1, 2)
    assert po.data_ptr() == ring.partial_out[2 * n + 1].data_ptr()
    # shards that are not back to back are refused, and so is the pass-KV driver
    swapped = [qs[1], qs[0]] + qs[2:]
    loose = B.Ring(swapped, kv[0], kv[1], qps, [i32(kp) for _, kp in sh],
                   out_dtype=torch.float32, keep_partials=True, gathered_q=True)
    with pytest.raises(B.CpError):
        B.cp_ring_passq(loose)
    with pytest.raises(B.CpError):
        B.cp_ring_passkv(ring)


def test_ring_passq_gathered_queries_decode(oracle):
    n, nh = 4, 16
    lengths = [900, 35, 2300, 1, 640, 1200, 77, 3000]
    ks = [W.normal(200 + b, (L, 1, 128)) for b, L in enumerate(lengths)]
    vs = [W.normal(300 + b, (L, 1, 128)) for b, L in enumerate(lengths)]
    qs = [W.normal(400 + b, (1, nh, 128)) for b in range(len(lengths))]
    ranks = oracle.shard_decode_batch(lengths, n, decode_iter=3)

    def gather(src, r):
        if len(r["kv_pos"]) == 0:
            return torch.zeros((0, 1, 128), dtype=torch.bfloat16)
        return torch.cat([src[b][p][None] for b, p in zip(r["kv_seq"], r["kv_pos"])])
    rk = [gather(ks, r) for r in ranks]
    rv = [gather(vs, r) for r in ranks]
    rq = [torch.cat([qs[b] for b in r["bid"]]) for r in ranks]
    ref_o, ref_l, _, _ = oracle.ring_passq_decode(
        [W.to_f64(x) for x in rq], [r["bid"] for r in ranks], [r["q_pos"] for r in ranks],
        [W.to_f64(x) for x in rk], [W.to_f64(x) for x in rv], [r["kv_pos"] for r in ranks],
        [r["cu_kv"] for r in ranks])
    m = len(ranks[0]["bid"])
    assert all(len(r["bid"]) == m for r in ranks)
    q_all = dev(torch.cat(rq))
    qpos_all = i32(np.concatenate([r["q_pos"] for r in ranks]))
    bid_all = i32(np.concatenate([r["bid"] for r in ranks]))
    sl = [slice(s * m, (s + 1) * m) for s in range(n)]
    for unique in (False, True):
        # unique: every holder's split partials stay in the workspace and one launch merges
        # over splits and holders together
        ring = B.Ring([q_all[x] for x in sl], [dev(x) for x in rk], [dev(x) for x in rv],
                      [qpos_all[x] for x in sl], [i32(r["kv_pos"]) for r in ranks],
                      out_dtype=torch.float32, keep_partials=True, gathered_q=True,
                      cu_seqlens_kv=[i32(r["cu_kv"]) for r in ranks],
                      bid=[bid_all[x] for x in sl], unique_bid=unique)
        out, lse = B.cp_ring_passq_decode(ring)
        torch.cuda.synchronize()
        for s in range(n):
            check(out[s], lse[s], ref_o[s], ref_l[s],
                  what="gathered decode, source %d, unique_bid %s" % (s, unique))


# ---------------------------------------------------------------------------
# ring drivers over packed batches (fused variable-length inputs of Algorithm 2)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("dtype,nh,nkv,d,lengths", [
    ("bf16", 16, 1, 128, [700, 5, 1300, 64, 2048]),
    ("bf16", 8, 2, 128, [333, 1, 900]),
    ("fp32", 4, 1, 64, [100, 3, 257]),
])
def test_ring_drivers_over_a_packed_batch(oracle, dtype, nh, nkv, d, lengths):
    n = 3
    qs = [randn(800 + b, (L, nh, d), dtype) for b, L in enumerate(lengths)]
    ks = [randn(820 + b, (L, nkv, d), dtype) for b, L in enumerate(lengths)]
    vs = [randn(840 + b, (L, nkv, d), dtype) for b, L in enumerate(lengths)]
    ref = [oracle.unsharded_causal(qs[b][1], ks[b][1], vs[b][1]) for b in range(len(lengths))]
    pos = [[B.cp_shard_positions(L, n, r) for L in lengths] for r in range(n)]
    cu = [np.concatenate([[0], np.cumsum([len(p) for p in pos[r]])]).astype(np.int32)
          for r in range(n)]

    def pack(src, r):
        return torch.cat([src[b][0][pos[r][b]] for b in range(len(lengths))])
    rq, rk, rv = ([pack(x, r) for r in range(n)] for x in (qs, ks, vs))
    rpos = [np.concatenate(pos[r]) for r in range(n)]
    atol, rtol = (2e-2, 1e-3) if dtype == "bf16" else (O_ATOL_FP32, LSE_RTOL_FP32)
    part_ref = oracle.ring_passkv([W.to_f64(x) for x in rq], [W.to_f64(x) for x in rk],
                                  [W.to_f64(x) for x in rv], rpos, rpos, cu_q=cu, cu_kv=cu)
    for order in (B.cp_ring_passkv, B.cp_ring_passq):
        for keep in (False, True):
            ring = B.Ring([dev(x) for x in rq], [dev(x) for x in rk], [dev(x) for x in rv],
                          [i32(p) for p in rpos], [i32(p) for p in rpos],
                          out_dtype=torch.float32, keep_partials=keep,
                          cu_seqlens_q=[i32(c) for c in cu], cu_seqlens_kv=[i32(c) for c in cu])
            out, lse = order(ring)
            torch.cuda.synchronize()
            for r in range(n):
                for b in range(len(lengths)):
                    sl = slice(cu[r][b], cu[r][b + 1])
                    check(out[r][sl], lse[r][sl], ref[b][0][pos[r][b]], ref[b][1][pos[r][b]],
                          o_atol=atol, lse_rtol=rtol,
                          what="%s rank %d sequence %d" % (order.__name__, r, b))
            if keep:   # the per-(rank, shard) partials too
                for a in range(n):
                    for s in range(n):
                        po, pl = ring.partial(a, s)
                        check(po, pl, part_ref[2][a][s], part_ref[3][a][s], o_atol=atol,
                              lse_rtol=rtol, what="partial %d,%d" % (a, s))
    with pytest.raises(B.CpError):   # the fused modes take one sequence only
        B.cp_ring_passkv(B.Ring([dev(x) for x in rq], [dev(x) for x in rk], [dev(x) for x in rv],
                                [i32(p) for p in rpos], [i32(p) for p in rpos], fused_merge=True,
                                cu_seqlens_q=[i32(c) for c in cu],
                                cu_seqlens_kv=[i32(c) for c in cu]))


def test_positions_close_to_the_int32_limit(oracle):
    """Positions are compared as int32: a sequence whose positions end two below the pad value
    behaves like the same sequence at zero (MFMA partial, decode, vector kernel)."""
    t, nh = 700, 16
    base = B.CP_POS_PAD_KV - 1 - t           # last position = INT32_MAX - 2
    q, q64 = randn(171, (t, nh, 128))
    k, k64 = randn(172, (t, 1, 128))
    v, v64 = randn(173, (t, 1, 128))
    rng = np.random.default_rng(3)
    kp = rng.permutation(t)
    qp = rng.integers(0, t, size=t)
    ref = oracle.attn(q64, k64, v64, qp, kp)
    o, l = gpu_partial(q, k, v, qp + base, kp + base, out_dtype=torch.float32)
    check(o, l, *ref, what="MFMA partial at the int32 limit")
    # decode: one query at the last position against the whole sequence
    od, ld = B.cp_attn_decode(dev(q[:1]), dev(k), dev(v), i32([base + t - 1]), i32(kp + base),
                              i32([0, t]), i32([0]), out_dtype=torch.float32)
    torch.cuda.synchronize()
    rd = oracle.attn(q64[:1], k64, v64, [t - 1], kp)
    check(od, ld, *rd, what="decode at the int32 limit")
    # fp32 vector kernel
    qf, qf64 = randn(174, (40, 4, 64), "fp32")
    kf, kf64 = randn(175, (90, 1, 64), "fp32")
    vf, vf64 = randn(176, (90, 1, 64), "fp32")
    qpf, kpf = rng.integers(0, 90, size=40), rng.permutation(90)
    big = B.CP_POS_PAD_KV - 1 - 90
    o, l = gpu_partial(qf, kf, vf, qpf + big, kpf + big, out_dtype=torch.float32)
    check(o, l, *oracle.attn(qf64, kf64, vf64, qpf, kpf), o_atol=O_ATOL_FP32,
          lse_rtol=LSE_RTOL_FP32, what="vector kernel at the int32 limit")


def test_ring_prefill_follows_the_selector(oracle):
    """cp_ring_prefill runs the order the selection rule picks: pass-Q for a small partial
    prefill behind a long cache, pass-KV for a full prefill; same exact result either way."""
    n, nh, d = 4, 16, 128
    for p_cached, t_new, expect in ((6000, 128, B.CP_ORDER_PASS_Q), (0, 2048, B.CP_ORDER_PASS_KV)):
        q, q64 = randn(181, (t_new, nh, d))
        k, k64 = randn(182, (p_cached + t_new, 1, d))
        v, v64 = randn(183, (p_cached + t_new, 1, d))
        ref_o, ref_l = oracle.unsharded_causal(q64, k64, v64, p_cached=p_cached)
        sh = oracle.shard_partial_prefill(p_cached, t_new, n)
        ring = B.Ring([dev(q[qp - p_cached]) for qp, _ in sh], [dev(k[kp]) for _, kp in sh],
                      [dev(v[kp]) for _, kp in sh], [i32(qp) for qp, _ in sh],
                      [i32(kp) for _, kp in sh], out_dtype=torch.float32)
        # Llama3-405B heads, an attention rate and a link for which Equation 2 gives T >= 5120
        out, lse, order = B.cp_ring_prefill(ring, p_cached, 128, 8, peak_flops=1.024e15,
                                            bandwidth=50e9)
        torch.cuda.synchronize()
        name = {B.CP_ORDER_PASS_KV: "pass-KV", B.CP_ORDER_PASS_Q: "pass-Q"}[order]
        assert order == expect
        assert name == oracle.select_order(t_new, p_cached, 128, 8, n, 1.024e15, 50e9)
        for r, (qp, _) in enumerate(sh):
            check(out[r], lse[r], ref_o[qp - p_cached], ref_l[qp - p_cached],
                  what="T %d rank %d" % (t_new, r))


def test_ring_walk_under_a_hip_graph(oracle):
    """The whole pass-KV ring (tile-bound pre-passes + one walk launch per rank) recorded in a
    HIP graph: the library enqueues kernels only, so every replay, with new Q written into the
    same buffers and eager work in between, equals the eager result bit for bit."""
    n, t = 4, 8192
    pos = [B.cp_shard_positions(t, n, r) for r in range(n)]
    k = W.normal(192, (t, 1, 128))
    v = W.normal(193, (t, 1, 128))
    qs_dev = [torch.zeros((len(p), 16, 128), dtype=torch.bfloat16, device="cuda") for p in pos]
    flags = [torch.ones(n, dtype=torch.int32, device="cuda") for _ in range(n)]
    ring = B.Ring(qs_dev, [dev(k[p]) for p in pos], [dev(v[p]) for p in pos],
                  [i32(p) for p in pos], [i32(p) for p in pos], out_dtype=torch.float32,
                  fused_merge=2, arrived=flags)
    inputs = [W.normal(194 + i, (t, 16, 128)) for i in range(3)]

    def stage(q):
        for r in range(n):
            qs_dev[r].copy_(q[pos[r]])
    eager = []
    for q in inputs:
        stage(q)
        B.cp_ring_passkv(ring)
        torch.cuda.synchronize()
        eager.append(([o.clone() for o in ring.out], [l.clone() for l in ring.lse]))
    # parity of the first input against the oracle on a few rows of rank 1
    rows = np.r_[0:8, 1020:1030, 2040:2048]
    tok = pos[1][rows]
    ref_o, ref_l = oracle.attn(W.to_f64(inputs[0][tok]), W.to_f64(k), W.to_f64(v), tok,
                               np.arange(t))
    check(eager[0][0][1][rows], eager[0][1][1][rows], ref_o, ref_l, what="eager, rank 1")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        g.capture_begin(capture_error_mode="relaxed")
        B.cp_ring_passkv(ring)
        g.capture_end()
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda")
    for i, q in enumerate(inputs):
        stage(q)
        scratch.add_(1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for r in range(n):
            assert torch.equal(ring.out[r], eager[i][0][r]), "replay %d rank %d" % (i, r)
            assert torch.equal(ring.lse[r], eager[i][1][r]), "replay %d rank %d" % (i, r)
    assert not ring.arrival_failed()
