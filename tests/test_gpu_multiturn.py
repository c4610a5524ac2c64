"""GPU parity for the persistent KV cache (Sections 3.5.2, 3.6): appends are compared slot by
slot with the oracle's cache, and a multi-turn replay (full prefill, decode steps with the
round-robin placement, a partial prefill, another decode step) is compared turn by turn with
causal attention over each sequence's whole history computed by the fp64 oracle."""
import numpy as np
import pytest
import torch

from gpu_util import check, dev, i32
from paper_2411_01783_amd import binding as B
from paper_2411_01783_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    B.load()  # raises if the HIP library is missing: no fallback
    assert torch.cuda.is_available()


def assert_cache_equals(cache: B.KVCache, ref, what=""):
    """Bit-exact: positions, K and V of every slot (unused ones hold zeros), used counts."""
    torch.cuda.synchronize()
    k_ref, v_ref, pos_ref, cu_ref = ref.packed()
    np.testing.assert_array_equal(cache.cu.cpu().numpy(), cu_ref, err_msg=what)
    used = cache.used.cpu().numpy()
    np.testing.assert_array_equal(used[:-1], ref.used(), err_msg=what)
    assert used[-1] == 0, what + ": the ticket word must be zero between calls"
    np.testing.assert_array_equal(cache.kv_pos.cpu().numpy(), pos_ref, err_msg=what)
    assert int(cache.dropped.item()) == ref.dropped, what
    np.testing.assert_array_equal(W.to_f64(cache.k.cpu()), k_ref, err_msg=what)
    np.testing.assert_array_equal(W.to_f64(cache.v.cpu()), v_ref, err_msg=what)


@pytest.mark.parametrize("dtype,nkv,d", [("bf16", 1, 128), ("fp32", 2, 64), ("bf16", 4, 8)])
def test_kv_append_matches_oracle_cache(oracle, dtype, nkv, d):
    rng = np.random.default_rng(7)
    n_seq = 37
    cap = rng.integers(0, 90, n_seq)
    cap[5] = 0
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    cache = B.KVCache(cap, nkv, d, dtype=tdt)
    ref = oracle.KVCache(cap, nkv, d)
    assert_cache_equals(cache, ref, "after reset")
    for call in range(6):
        # some calls overflow some sequences on purpose (host-checked, in-bounds: dropped)
        counts = rng.integers(0, 40 if call < 4 else 3, n_seq)
        if call == 2:
            counts[:] = 0
            counts[11] = 1   # a single token, as a decode step appends
        if call == 3:
            counts[:] = 0    # nothing at all
        cu_new = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        total = int(cu_new[-1])
        k_new = W.normal(100 + call, (total, nkv, d), dtype)
        v_new = W.normal(200 + call, (total, nkv, d), dtype)
        pos_new = rng.integers(0, 1 << 20, total).astype(np.int32)
        B.cp_kv_append(cache, dev(k_new), dev(v_new), i32(pos_new), i32(cu_new))
        for b in range(n_seq):
            sl = slice(cu_new[b], cu_new[b + 1])
            ref.append(b, W.to_f64(k_new[sl]), W.to_f64(v_new[sl]), pos_new[sl])
        assert_cache_equals(cache, ref, "after call %d" % call)
    assert ref.dropped > 0  # the overflow path was exercised


def test_multi_turn_replay(oracle):
    n, nh, d = 4, 16, 128
    first, second = [700, 260, 1500, 33], [300, 1024, 17, 256]
    n_seq = len(first)
    n_decode = n + 1
    total = [a + b + n_decode + 1 for a, b in zip(first, second)]
    cap = [-(-(a + b) // n) + n_decode + 5 for a, b in zip(first, second)]
    qs = [W.normal(600 + b, (total[b], nh, d)) for b in range(n_seq)]
    ks = [W.normal(620 + b, (total[b], 1, d)) for b in range(n_seq)]
    vs = [W.normal(640 + b, (total[b], 1, d)) for b in range(n_seq)]
    ref = [oracle.unsharded_causal(W.to_f64(qs[b]), W.to_f64(ks[b]), W.to_f64(vs[b]))
           for b in range(n_seq)]
    caches = [B.KVCache(cap, 1, d) for _ in range(n)]
    ref_caches = [oracle.KVCache(cap, 1, d) for _ in range(n)]
    length = [0] * n_seq

    def append(r, b, pos):
        pos = np.asarray(pos, dtype=np.int64)
        cu_new = np.zeros(n_seq + 1, dtype=np.int32)
        cu_new[b + 1:] = len(pos)
        B.cp_kv_append(caches[r], dev(ks[b][pos]), dev(vs[b][pos]), i32(pos), i32(cu_new))
        ref_caches[r].append(b, W.to_f64(ks[b][pos]), W.to_f64(vs[b][pos]), pos)

    def prefill_turn(b, t_new, order, what):
        p0 = length[b]
        qpos = [B.cp_shard_positions(t_new, n, r, offset=p0) for r in range(n)]
        for r in range(n):
            append(r, b, qpos[r])      # KV_k of Algorithms 2 / 3: the cache plus this turn's K/V
        seg = [caches[r].segment(b) for r in range(n)]
        ring = B.Ring([dev(qs[b][p]) for p in qpos], [s[0] for s in seg], [s[1] for s in seg],
                      [i32(p) for p in qpos], [s[2] for s in seg], out_dtype=torch.float32)
        out, lse = order(ring)
        torch.cuda.synchronize()
        for r in range(n):
            check(out[r], lse[r], ref[b][0][qpos[r]], ref[b][1][qpos[r]],
                  what="%s seq %d rank %d" % (what, b, r))
        length[b] += t_new

    def decode_turn(t):
        bids = [[] for _ in range(n)]
        for b in range(n_seq):
            r = B.cp_decode_owner(b, t, n)
            assert r == oracle.decode_owner(b, t, n)
            append(r, b, [length[b]])
            bids[r].append(b)
        rq = [torch.cat([qs[b][length[b]:length[b] + 1] for b in bs]) if bs else
              torch.zeros((0, nh, d), dtype=torch.bfloat16) for bs in bids]
        ring = B.Ring([dev(x) for x in rq], [c.k for c in caches], [c.v for c in caches],
                      [i32([length[b] for b in bs]) for bs in bids], [c.kv_pos for c in caches],
                      out_dtype=torch.float32, cu_seqlens_kv=[c.cu for c in caches],
                      bid=[i32(bs) for bs in bids])
        out, lse = B.cp_ring_passq_decode(ring)
        torch.cuda.synchronize()
        for r in range(n):
            for i, b in enumerate(bids[r]):
                p = length[b]
                check(out[r][i:i + 1], lse[r][i:i + 1], ref[b][0][p:p + 1], ref[b][1][p:p + 1],
                      what="decode iteration %d seq %d" % (t, b))
        for b in range(n_seq):
            length[b] += 1

    for b in range(n_seq):
        prefill_turn(b, first[b], B.cp_ring_passkv, "full prefill")
    for t in range(n_decode):
        decode_turn(t)
    for b in range(n_seq):
        prefill_turn(b, second[b], B.cp_ring_passq if b % 2 else B.cp_ring_passkv,
                     "partial prefill")
    decode_turn(n_decode)
    assert length == total
    for r in range(n):
        assert_cache_equals(caches[r], ref_caches[r], "rank %d cache after the last turn" % r)
        assert ref_caches[r].dropped == 0


def test_decode_step_under_a_hip_graph(oracle):
    """A decode step (append of the new tokens' K/V on their owners, then the pass-Q decode
    ring) recorded once and replayed: every replay, with new queries and new K/V written into
    the same input buffers and eager work in between, matches the eager result bit for bit and
    the oracle within the bars; the caches grow by one token per sequence per replay."""
    n, nh, d, n_seq, n_steps = 4, 16, 128, 8, 4
    first = [300, 31, 1200, 64, 513, 5, 777, 128]
    cap = [-(-L // n) + n_steps + 2 for L in first]
    total = [L + n_steps for L in first]
    qs = [W.normal(700 + b, (total[b], nh, d)) for b in range(n_seq)]
    ks = [W.normal(720 + b, (total[b], 1, d)) for b in range(n_seq)]
    vs = [W.normal(740 + b, (total[b], 1, d)) for b in range(n_seq)]
    ref = [oracle.unsharded_causal(W.to_f64(qs[b]), W.to_f64(ks[b]), W.to_f64(vs[b]))
           for b in range(n_seq)]

    def fresh_caches():
        caches = [B.KVCache(cap, 1, d) for _ in range(n)]
        for b in range(n_seq):
            for r in range(n):
                pos = B.cp_shard_positions(first[b], n, r).astype(np.int64)
                cu_new = np.zeros(n_seq + 1, dtype=np.int32)
                cu_new[b + 1:] = len(pos)
                B.cp_kv_append(caches[r], dev(ks[b][pos]), dev(vs[b][pos]), i32(pos), i32(cu_new))
        return caches

    # With n_seq a multiple of n every rank owns n_seq / n tokens at every iteration, so the
    # shapes of a step do not change; which sequences they are does (round-robin), and that
    # lives in device buffers the graph reads: bid, q_pos, cu_seqlens_new, the new rows.
    per = n_seq // n
    bufs = [dict(q=torch.zeros((per, nh, d), dtype=torch.bfloat16, device="cuda"),
                 k=torch.zeros((per, 1, d), dtype=torch.bfloat16, device="cuda"),
                 v=torch.zeros((per, 1, d), dtype=torch.bfloat16, device="cuda"),
                 pos=torch.zeros(per, dtype=torch.int32, device="cuda"),
                 bid=torch.zeros(per, dtype=torch.int32, device="cuda"),
                 cu_new=torch.zeros(n_seq + 1, dtype=torch.int32, device="cuda"))
            for _ in range(n)]

    def stage(t):
        owned = [[b for b in range(n_seq) if B.cp_decode_owner(b, t, n) == r] for r in range(n)]
        for r in range(n):
            bs = owned[r]
            p = [first[b] + t for b in bs]
            bufs[r]["q"].copy_(torch.cat([qs[b][x:x + 1] for b, x in zip(bs, p)]))
            bufs[r]["k"].copy_(torch.cat([ks[b][x:x + 1] for b, x in zip(bs, p)]))
            bufs[r]["v"].copy_(torch.cat([vs[b][x:x + 1] for b, x in zip(bs, p)]))
            bufs[r]["pos"].copy_(i32(p))
            bufs[r]["bid"].copy_(i32(bs))
            counts = np.zeros(n_seq, dtype=np.int64)
            counts[bs] = 1
            bufs[r]["cu_new"].copy_(i32(np.concatenate([[0], np.cumsum(counts)])))
        return owned

    def make_step(caches):
        ring = B.Ring([x["q"] for x in bufs], [c.k for c in caches], [c.v for c in caches],
                      [x["pos"] for x in bufs], [c.kv_pos for c in caches],
                      out_dtype=torch.float32, cu_seqlens_kv=[c.cu for c in caches],
                      bid=[x["bid"] for x in bufs])

        def step():
            for r in range(n):
                B.cp_kv_append(caches[r], bufs[r]["k"], bufs[r]["v"], bufs[r]["pos"],
                               bufs[r]["cu_new"])
            B.cp_ring_passq_decode(ring)
        return ring, step

    # eager run: the expected outputs of every step
    caches = fresh_caches()
    ring, step = make_step(caches)
    eager = []
    for t in range(n_steps):
        owned = stage(t)
        step()
        torch.cuda.synchronize()
        eager.append(([o.clone() for o in ring.out], [l.clone() for l in ring.lse]))
        for r in range(n):
            for i, b in enumerate(owned[r]):
                p = first[b] + t
                check(ring.out[r][i:i + 1], ring.lse[r][i:i + 1], ref[b][0][p:p + 1],
                      ref[b][1][p:p + 1], what="eager step %d seq %d" % (t, b))
    eager_used = [c.used.cpu().numpy().copy() for c in caches]

    # the same steps from one graph over fresh caches
    caches = fresh_caches()
    ring, step = make_step(caches)
    stage(0)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        g.capture_begin(capture_error_mode="relaxed")
        step()
        g.capture_end()
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda")
    for t in range(n_steps):
        stage(t)                       # eager copies into the graph's input buffers
        scratch.add_(1.0)              # unrelated eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for r in range(n):
            assert torch.equal(ring.out[r], eager[t][0][r]), "replay %d rank %d" % (t, r)
            assert torch.equal(ring.lse[r], eager[t][1][r]), "replay %d rank %d" % (t, r)
    for r in range(n):
        np.testing.assert_array_equal(caches[r].used.cpu().numpy(), eager_used[r])
        assert int(caches[r].dropped.item()) == 0
        assert caches[r].used.cpu().numpy()[:-1].sum() == \
            sum(len(B.cp_shard_positions(L, n, r)) for L in first) + n_steps * per
