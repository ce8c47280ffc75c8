"""Measurement aids of bench.py that are no part of the CSAttention library: built as a library of
their own (librow_gather_probe.so) next to their source."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "row_gather_probe.hip")
LIB = os.path.join(HERE, "librow_gather_probe.so")
_lib = None


def build(verbose: bool = True) -> str:
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
           "-shared", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", SRC, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def probe_row_gather(k_rows, v_rows, idx, check):
    """k_rows, v_rows: [n_rows][128] bf16 device tensors; idx: int32 [n_idx]; check: 32-bit
    [ceil(n_idx / 64)].  Launches on torch's current stream."""
    import torch
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise RuntimeError(f"{LIB} is missing: build it with __graft_entry__.build()")
        _lib = C.CDLL(LIB)
        _lib.probe_row_gather.restype = C.c_int
        _lib.probe_row_gather.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                          C.c_void_p]
    n_rows = k_rows.numel() // 128
    assert v_rows.numel() // 128 == n_rows and k_rows.element_size() == 2 and idx.dtype == torch.int32
    assert check.element_size() == 4 and check.numel() >= (idx.numel() + 63) // 64
    for t in (k_rows, v_rows, idx, check):
        assert t.is_cuda and t.is_contiguous()
    rc = _lib.probe_row_gather(k_rows.data_ptr(), v_rows.data_ptr(), n_rows, idx.data_ptr(), idx.numel(),
                               check.data_ptr(), torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"probe_row_gather failed ({rc})")
