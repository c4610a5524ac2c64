"""cp_attn_decode_static (the entry point that allocates nothing) against cp_attn_decode.

Both run the same kernels; the only difference is where the split-KV partials live (the
library's own scratch array instead of a caller's workspace), so the results must be equal
bit for bit. Two calls in a row, the second on a smaller input: the scratch keeps the first
call's contents, which the second must not pick up."""
import numpy as np
import pytest
import torch

from paper_2411_01783_amd import binding as B
from gpu_util import check, dev, i32, randn

pytestmark = pytest.mark.gpu


def _case(lengths, bid, seed, nh=16, nkv=1, d=128):
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    total = int(cu[-1])
    q, q64 = randn(seed, (len(bid), nh, d))
    k, k64 = randn(seed + 1, (total, nkv, d))
    v, v64 = randn(seed + 2, (total, nkv, d))
    kp = np.concatenate([np.arange(L) for L in lengths]).astype(np.int32)
    qp = np.array([lengths[b] - 1 for b in bid], dtype=np.int32)
    return dict(q=dev(q), k=dev(k), v=dev(v), qp=i32(qp), kp=i32(kp), cu=i32(cu), bid=i32(bid),
                host=(q64, k64, v64, qp, kp, cu, np.asarray(bid)))


def test_decode_static_equals_decode_on_two_calls_in_a_row(oracle):
    B.load()
    big = _case([4097, 2500, 8192, 700, 3000, 129, 6000, 5000], [0, 1, 2, 3, 4, 5, 6, 7], 501)
    small = _case([300, 31, 1000], [2, 0], 511)
    for what, c in (("first call", big), ("second, smaller call", small)):
        nq = c["q"].shape[0]
        # (both decode paths: split per query, and flat key ranges under CP_SHAPE_UNIQUE_BID)
        for odt, unique in ((torch.float32, False), (torch.bfloat16, False), (torch.float32, True)):
            ref_o, ref_l = B.cp_attn_decode(c["q"], c["k"], c["v"], c["qp"], c["kp"], c["cu"],
                                            c["bid"], out_dtype=odt, unique_bid=unique)
            out = torch.full((nq, 16, 128), float("nan"), dtype=odt, device="cuda")
            lse = torch.full((nq, 16), float("nan"), dtype=torch.float32, device="cuda")
            B.cp_attn_decode_static(c["q"], c["k"], c["v"], c["qp"], c["kp"], c["cu"], c["bid"],
                                    out, lse, unique_bid=unique)
            torch.cuda.synchronize()
            assert torch.equal(out, ref_o), what
            assert torch.equal(lse, ref_l), what
        # and against the oracle, to the same bar as cp_attn_decode's own tests
        q64, k64, v64, qp, kp, cu, bid = c["host"]
        ro = np.zeros((nq, 16, 128))
        rl = np.zeros((nq, 16))
        for i, b in enumerate(bid):
            o1, l1 = oracle.attn(q64[i:i + 1], k64[cu[b]:cu[b + 1]], v64[cu[b]:cu[b + 1]],
                                 qp[i:i + 1], kp[cu[b]:cu[b + 1]])
            ro[i], rl[i] = o1[0], l1[0]
        check(out.float(), lse, ro, rl, what="static decode, " + what)
