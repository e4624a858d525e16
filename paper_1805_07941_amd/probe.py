"""ctypes binding of libdfq_probe.so (include/dfq_probe.h): a measurement aid for benchmarks, not part
of the quantized path."""
from __future__ import annotations

import ctypes as C
import os

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdfq_probe.so")
EXPORTS = ["dfq_probe_item_loop_rate", "dfq_probe_mfma_rate"]
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1805_07941_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.dfq_probe_mfma_rate.restype = C.c_int
        L.dfq_probe_mfma_rate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_double), C.c_void_p]
        L.dfq_probe_item_loop_rate.restype = C.c_int
        L.dfq_probe_item_loop_rate.argtypes = L.dfq_probe_mfma_rate.argtypes
        _lib = L
    return _lib


def item_loop_rate(a_codes: torch.Tensor, b_codes: torch.Tensor, sink: torch.Tensor, blocks: int, steps: int, stream=None) -> float:
    """Launches the dense kernel's item pipeline without global loads (matrix instructions, barrier, LDS reads) on the
    operand bytes; returns the number of operations of the launch.  The caller times it."""
    return _launch("dfq_probe_item_loop_rate", a_codes, b_codes, sink, blocks, steps, stream)


def mfma_rate(a_codes: torch.Tensor, b_codes: torch.Tensor, sink: torch.Tensor, blocks: int, iters: int, stream=None) -> float:
    """Launches the register-only matrix-instruction loop on operand bytes taken from ``a_codes`` (first
    16 KiB) and ``b_codes`` (first 32 KiB); returns the number of operations of the launch.  The caller
    times it."""
    return _launch("dfq_probe_mfma_rate", a_codes, b_codes, sink, blocks, iters, stream)


def _launch(name, a_codes, b_codes, sink, blocks, iters, stream):
    for t, dt in ((a_codes, torch.int8), (b_codes, torch.int8), (sink, torch.int32)):
        if not t.is_cuda or t.dtype != dt or not t.is_contiguous():
            raise TypeError("probe: contiguous CUDA tensors (int8, int8, int32)")
    if a_codes.numel() < 16384 or b_codes.numel() < 32768 or sink.numel() < blocks * 512:
        raise ValueError("probe: a_codes >= 16 KiB, b_codes >= 32 KiB, sink >= blocks * 512 words")
    st = torch.cuda.current_stream().cuda_stream if stream is None else (stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))
    ops = C.c_double(0.0)
    rc = getattr(lib(), name)(a_codes.data_ptr(), b_codes.data_ptr(), sink.data_ptr(), int(blocks), int(iters), C.byref(ops), st)
    if rc != 0:
        raise RuntimeError(f"{name}: status {rc}")
    return ops.value
