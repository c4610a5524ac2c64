"""Builds and loads libbench_probes.so (bench_probes.hip): a bare MFMA loop and a bare
streaming read, the yardsticks bench.py reports beside the kernels' own figures."""
from __future__ import annotations

import ctypes
import os
import subprocess

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bench_probes.hip")
LIB = os.path.join(HERE, "libbench_probes.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
OPERAND_BYTES = 65536

_lib = None


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", SRC, "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (SRC, res.stderr))
    os.replace(tmp, LIB)
    return LIB


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise RuntimeError("libbench_probes.so not built: run __graft_entry__.build()")
        lib = ctypes.CDLL(LIB)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.bench_probe_hbm_read.restype = ctypes.c_int
        lib.bench_probe_hbm_read.argtypes = [vp, ctypes.c_size_t, i32, vp, vp]
        lib.bench_probe_mfma_rate.restype = ctypes.c_int
        lib.bench_probe_mfma_rate.argtypes = [vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        _lib = lib
    return _lib


def mfma_rate(operands: torch.Tensor, iters: int, n_workgroups: int, sink: torch.Tensor) -> float:
    """Launch the matrix-pipe rate probe on torch's current stream; returns the launch's FLOPs."""
    assert operands.numel() * operands.element_size() >= OPERAND_BYTES
    assert sink.numel() >= n_workgroups * 512 and sink.dtype == torch.float32
    flop = ctypes.c_double(0.0)
    rc = load().bench_probe_mfma_rate(operands.data_ptr(), int(iters), int(n_workgroups),
                                      sink.data_ptr(), ctypes.byref(flop),
                                      torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("bench_probe_mfma_rate failed (%d)" % rc)
    return flop.value


def hbm_read(buffer: torch.Tensor, n_workgroups: int, sink: torch.Tensor) -> int:
    """One streaming read of the whole buffer on torch's current stream; returns the bytes read."""
    nbytes = buffer.numel() * buffer.element_size()
    if sink.numel() * sink.element_size() < n_workgroups * 256 * 4:
        raise ValueError("sink too small")
    rc = load().bench_probe_hbm_read(buffer.data_ptr(), nbytes, n_workgroups, sink.data_ptr(),
                                     torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("bench_probe_hbm_read failed (%d)" % rc)
    return nbytes
