"""SPARQ CPU oracle -- TEST INFRASTRUCTURE ONLY.

ctypes front end of ``sparq_oracle.c`` (plain C, host pointers).  Only the
tests, the smoke check and the CPU-baseline leg of the benchmark may import
this package; the GPU library never does, and the two share no code.

The C file follows the paper step by step: bSPARQ window placement and
rounding (Section 3.1), the vSPARQ pair rule (Section 3.2, Eq. 2), the integer
dot product of Eq. 1 laid out as a convolution, and the per-output-channel
dequantisation and the requantisation to unsigned 8 bits implied by the
quantisation scheme of Section 5.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparq_oracle.c")
_LIB = os.path.join(_HERE, "libsparq_oracle.so")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


class Mode(ctypes.Structure):
    _fields_ = [("window_bits", ctypes.c_int32), ("shift_mask", ctypes.c_uint32),
                ("round_nearest", ctypes.c_int32), ("pair", ctypes.c_int32)]


class Conv(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in
                ("B", "H", "W", "C", "N", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w")]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        L.sparq_ref_mode_check.argtypes = [ctypes.POINTER(Mode)]
        L.sparq_ref_mode_check.restype = ctypes.c_int
        L.sparq_ref_wide_shift_mask.argtypes = [ctypes.c_int32, ctypes.c_uint32]
        L.sparq_ref_wide_shift_mask.restype = ctypes.c_uint32
        L.sparq_ref_trim_value.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_uint32, ctypes.c_int,
                                           ctypes.POINTER(ctypes.c_int)]
        L.sparq_ref_trim_value.restype = ctypes.c_int
        L.sparq_trim_ref.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                     ctypes.POINTER(Mode)]
        L.sparq_trim_ref.restype = ctypes.c_int
        L.sparq_conv_gemm_ref.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(Conv),
                                          ctypes.POINTER(Mode), ctypes.c_void_p, ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.sparq_conv_gemm_ref.restype = ctypes.c_int
        L.sparq_dequant_ref.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_int32]
        L.sparq_dequant_ref.restype = ctypes.c_int
        L.sparq_requant_ref.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_int32]
        L.sparq_requant_ref.restype = ctypes.c_int
        L.sparq_conv_gemm_sparse24_ref.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(Conv),
                                                   ctypes.POINTER(Mode), ctypes.c_void_p, ctypes.c_int64,
                                                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.sparq_conv_gemm_sparse24_ref.restype = ctypes.c_int
        L.sparq_ref_packed_record_bytes.argtypes = [ctypes.POINTER(Mode), ctypes.c_int32]
        L.sparq_ref_packed_record_bytes.restype = ctypes.c_int32
        L.sparq_pack_act_ref.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                         ctypes.POINTER(Mode), ctypes.c_int32]
        L.sparq_pack_act_ref.restype = ctypes.c_int
        L.sparq_unpack_act_ref.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                           ctypes.POINTER(Mode), ctypes.c_int32]
        L.sparq_unpack_act_ref.restype = ctypes.c_int
        _lib = L
    return _lib


def _mode(window_bits=4, shift_mask=0x1F, round_nearest=0, pair=1) -> Mode:
    return Mode(int(window_bits), int(shift_mask), int(round_nearest), int(pair))


def mode_check(window_bits, shift_mask, round_nearest, pair) -> int:
    m = _mode(window_bits, shift_mask, round_nearest, pair)
    return lib().sparq_ref_mode_check(ctypes.byref(m))


def wide_shift_mask(n: int, shift_mask: int) -> int:
    return int(lib().sparq_ref_wide_shift_mask(n, shift_mask))


def trim_value(x: int, n: int, shift_mask: int, round_nearest: int):
    """bSPARQ on one value -> (trimmed value, shift)."""
    s = ctypes.c_int(0)
    v = lib().sparq_ref_trim_value(int(x), int(n), int(shift_mask), int(round_nearest), ctypes.byref(s))
    return int(v), int(s.value)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def trim(x: np.ndarray, window_bits=4, shift_mask=0x1F, round_nearest=0, pair=1) -> np.ndarray:
    """vSPARQ+bSPARQ along the last axis of a uint8 array."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    C = x.shape[-1]
    rows = x.size // C if C else 0
    y = np.empty_like(x)
    m = _mode(window_bits, shift_mask, round_nearest, pair)
    rc = lib().sparq_trim_ref(_ptr(x), _ptr(y), rows, C, ctypes.byref(m))
    if rc:
        raise ValueError(f"sparq_trim_ref rejected its arguments (code {rc})")
    return y


def conv_out_hw(H, W, KH, KW, stride=(1, 1), pad=(0, 0)):
    return ((H + 2 * pad[0] - KH) // stride[0] + 1, (W + 2 * pad[1] - KW) // stride[1] + 1)


def conv_gemm(x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0), *, window_bits=4,
              shift_mask=0x1F, round_nearest=0, pair=1, scale=None, rows=None):
    """Trimmed convolution by definition.

    x uint8 [B,H,W,C]; w int8 [N,KH,KW,C]; returns (acc int32 [M or len(rows), N],
    out float64 or None).  ``rows`` selects output rows m=(b*Ho+oy)*Wo+ox.
    """
    x = np.ascontiguousarray(x, dtype=np.uint8)
    w = np.ascontiguousarray(w, dtype=np.int8)
    B, H, W, C = x.shape
    N, KH, KW, C2 = w.shape
    assert C2 == C
    d = Conv(B, H, W, C, N, KH, KW, stride[0], stride[1], pad[0], pad[1])
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    M = B * Ho * Wo
    ridx = None
    nr = M
    if rows is not None:
        ridx = np.ascontiguousarray(rows, dtype=np.int64)
        nr = ridx.size
    acc = np.empty((nr, N), dtype=np.int32)
    out = None
    sc = None
    if scale is not None:
        sc = np.ascontiguousarray(scale, dtype=np.float32)
        assert sc.shape == (N,)
        out = np.empty((nr, N), dtype=np.float64)
    m = _mode(window_bits, shift_mask, round_nearest, pair)
    rc = lib().sparq_conv_gemm_ref(_ptr(x), _ptr(w), ctypes.byref(d), ctypes.byref(m), _ptr(ridx), nr,
                                   _ptr(acc), _ptr(sc), _ptr(out))
    if rc:
        raise ValueError(f"sparq_conv_gemm_ref failed (code {rc})")
    return acc, out


def dequant(acc: np.ndarray, scale: np.ndarray) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    M, N = acc.shape
    out = np.empty((M, N), dtype=np.float64)
    rc = lib().sparq_dequant_ref(_ptr(acc), _ptr(scale), _ptr(out), M, N)
    if rc:
        raise ValueError(f"sparq_dequant_ref rejected its arguments (code {rc})")
    return out


def requant(acc: np.ndarray, factor: np.ndarray) -> np.ndarray:
    """y = clamp(rint(float32(acc) * factor[n]), 0, 255) as uint8 (Section 5: unsigned per-layer activations)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    factor = np.ascontiguousarray(factor, dtype=np.float32)
    M, N = acc.shape
    y = np.empty((M, N), dtype=np.uint8)
    rc = lib().sparq_requant_ref(_ptr(acc), _ptr(factor), _ptr(y), M, N)
    if rc:
        raise ValueError(f"sparq_requant_ref rejected its arguments (code {rc})")
    return y


def conv_gemm_u8(x: np.ndarray, w: np.ndarray, factor: np.ndarray, stride=(1, 1), pad=(0, 0), *, rows=None,
                 out_mode=None, **mode):
    """The trimmed convolution followed by the requantisation of its int32 result: uint8 [M or len(rows), N].
    out_mode (a dict of trim() keywords) trims the bytes as the next layer would: pairs along the N channels of a row."""
    acc, _ = conv_gemm(x, w, stride, pad, rows=rows, **mode)
    y = requant(acc, factor)
    return trim(y, **out_mode) if out_mode else y



def packed_record_bytes(group: int = 1, **mode) -> int:
    """Bytes of one 32-channel record of the packed form (Sections 3.1, 5.1, 6); 0 if the mode cannot be packed."""
    m = _mode(**mode)
    return int(lib().sparq_ref_packed_record_bytes(ctypes.byref(m), int(group)))


def pack_act(x: np.ndarray, group: int = 1, **mode) -> np.ndarray:
    """Packed records of the trimmed activations along the last axis of x: uint8 [rows, ceil(C/32) * record bytes]."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    C = x.shape[-1]
    rows = x.size // C
    rec = packed_record_bytes(group, **mode)
    if rec == 0:
        raise ValueError("this mode / group has no packed form")
    packed = np.empty((rows, (C + 31) // 32 * rec), dtype=np.uint8)
    m = _mode(**mode)
    rc = lib().sparq_pack_act_ref(_ptr(x), _ptr(packed), rows, C, ctypes.byref(m), int(group))
    if rc:
        raise ValueError(f"sparq_pack_act_ref rejected its arguments (code {rc})")
    return packed


def unpack_act(packed: np.ndarray, shape, group: int = 1, **mode) -> np.ndarray:
    """The uint8 tensor of `shape` the packed records encode."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    C = int(shape[-1])
    rows = int(np.prod(shape)) // C
    y = np.empty(shape, dtype=np.uint8)
    m = _mode(**mode)
    rc = lib().sparq_unpack_act_ref(_ptr(packed), _ptr(y), rows, C, ctypes.byref(m), int(group))
    if rc:
        raise ValueError(f"sparq_unpack_act_ref rejected its arguments (code {rc})")
    return y


def conv_gemm_sparse24(x: np.ndarray, w_vals: np.ndarray, w_idx: np.ndarray, stride=(1, 1), pad=(0, 0), *, scale=None,
                       rows=None, **mode):
    """Convolution with 2:4 pruned weights (Section 4, sparse tensor core): w_vals int8 / w_idx uint8 [N,KH,KW,C/2];
    the two activations an output channel's coordinates pick from a group of four form its vSPARQ pair.
    Returns (acc int32, out float64 or None) like conv_gemm."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    w_vals = np.ascontiguousarray(w_vals, dtype=np.int8)
    w_idx = np.ascontiguousarray(w_idx, dtype=np.uint8)
    B, H, W, C = x.shape
    N, KH, KW, C2 = w_vals.shape
    assert 2 * C2 == C and w_idx.shape == w_vals.shape
    d = Conv(B, H, W, C, N, KH, KW, stride[0], stride[1], pad[0], pad[1])
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    ridx, nr = None, B * Ho * Wo
    if rows is not None:
        ridx = np.ascontiguousarray(rows, dtype=np.int64)
        nr = ridx.size
    acc = np.empty((nr, N), dtype=np.int32)
    out = sc = None
    if scale is not None:
        sc = np.ascontiguousarray(scale, dtype=np.float32)
        out = np.empty((nr, N), dtype=np.float64)
    m = _mode(**mode)
    rc = lib().sparq_conv_gemm_sparse24_ref(_ptr(x), _ptr(w_vals), _ptr(w_idx), ctypes.byref(d), ctypes.byref(m),
                                            _ptr(ridx), nr, _ptr(acc), _ptr(sc), _ptr(out))
    if rc:
        raise ValueError(f"sparq_conv_gemm_sparse24_ref failed (code {rc})")
    return acc, out
