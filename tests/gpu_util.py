"""Helpers shared by the GPU parity tests: tolerance checks and oracle/GPU plumbing."""
import json
import os

import numpy as np
import torch

from paper_2411_01783_amd import workloads as W

# Tolerances for bf16 inputs with unit-scale values: max-abs 2e-2 on outputs,
# 1e-3 relative on LSE read as |d| <= 1e-3 * max(1, |LSE|); -inf must match exactly.
O_ATOL_BF16 = 2e-2
LSE_RTOL = 1e-3
# fp32 inputs through the fp32 vector kernel: rounding of fp32 dot products of length d
# and of exp/log approximations, well under 1e-4 for unit-scale inputs.
O_ATOL_FP32 = 1e-4
LSE_RTOL_FP32 = 1e-5


def dev(x, dtype=None):
    t = torch.as_tensor(x)
    if dtype is not None:
        t = t.to(dtype)
    return t.to("cuda").contiguous()


def i32(x):
    return torch.as_tensor(np.asarray(x, dtype=np.int32)).to("cuda")


def check(out, lse, ref_o, ref_l, o_atol=O_ATOL_BF16, lse_rtol=LSE_RTOL, what=""):
    """Element-by-element comparison of a GPU (O, LSE) with the oracle's."""
    o = out.detach().to("cpu", torch.float64).numpy()
    l = lse.detach().to("cpu", torch.float64).numpy()
    assert o.shape == ref_o.shape and l.shape == ref_l.shape, what
    assert not np.isnan(o).any() and not np.isnan(l).any(), what + ": NaN in output"
    empty = np.isneginf(ref_l)
    assert np.array_equal(np.isneginf(l), empty), what + ": -inf pattern of LSE differs"
    assert np.all(o[empty] == 0), what + ": rows without keys must be exactly zero"
    err_o = np.abs(o - ref_o).max() if o.size else 0.0
    assert err_o <= o_atol, "%s: max-abs O error %.3e > %.1e" % (what, err_o, o_atol)
    fin = ~empty
    rel_l = 0.0
    if fin.any():
        tol = lse_rtol * np.maximum(1.0, np.abs(ref_l[fin]))
        err_l = np.abs(l[fin] - ref_l[fin])
        rel_l = float((err_l / np.maximum(1.0, np.abs(ref_l[fin]))).max())
        assert np.all(err_l <= tol), "%s: LSE error %.3e" % (what, (err_l / tol).max() * lse_rtol)
    log = os.environ.get("CP_PARITY_LOG")
    if log:  # measured errors of every comparison, one JSON line each (for the results table)
        with open(log, "a") as f:
            f.write(json.dumps({"test": os.environ.get("PYTEST_CURRENT_TEST", ""), "what": what,
                                "rows": int(l.size), "max_abs_o": float(err_o),
                                "max_rel_lse": rel_l}) + "\n")
    return err_o


def rel_l2(out, ref_o):
    o = out.detach().to("cpu", torch.float64).numpy()
    den = np.linalg.norm(ref_o)
    return float(np.linalg.norm(o - ref_o) / den) if den > 0 else 0.0


def randn(seed, shape, dtype="bf16"):
    """Seeded N(0,1) in the storage dtype on the CPU; returns (torch tensor, exact fp64 copy)."""
    t = W.normal(seed, shape, dtype, "cpu")
    return t, W.to_f64(t)
