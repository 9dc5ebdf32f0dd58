"""ctypes binding of libsparq_probe.so (include/sparq_probe.h): the machine-ceiling micro-benchmarks the
benchmark reports next to the published peaks.  Marshalling only; torch provides device buffers and streams."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparq_probe.so")
OPERAND_BYTES = 12 * 256 * 16
SINK_BYTES = 256 * 256 * 4


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    vp = ctypes.c_void_p
    L.sparq_probe_mfma_i8_ops.argtypes = [ctypes.c_int32]
    L.sparq_probe_mfma_i8_ops.restype = ctypes.c_double
    L.sparq_probe_mfma_i8.argtypes = [vp, vp, ctypes.c_int32, vp]
    L.sparq_probe_mfma_i8.restype = ctypes.c_int
    L.sparq_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.sparq_probe_copy.restype = ctypes.c_int
    return L


lib = _load()


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def sparq_probe_mfma_i8_ops(iters: int) -> float:
    return float(lib.sparq_probe_mfma_i8_ops(int(iters)))


def sparq_probe_mfma_i8(operands: torch.Tensor, sink: torch.Tensor, iters: int) -> None:
    if operands.numel() * operands.element_size() < OPERAND_BYTES or sink.numel() * sink.element_size() < SINK_BYTES:
        raise ValueError("operand / sink buffer too small")
    rc = lib.sparq_probe_mfma_i8(operands.data_ptr(), sink.data_ptr(), int(iters), _stream())
    if rc:
        raise RuntimeError(f"sparq_probe_mfma_i8 failed (status {rc})")


def sparq_probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n:
        raise ValueError("size mismatch")
    rc = lib.sparq_probe_copy(src.data_ptr(), dst.data_ptr(), n, _stream())
    if rc:
        raise RuntimeError(f"sparq_probe_copy failed (status {rc})")
