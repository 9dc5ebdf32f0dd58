"""ctypes binding of libsparq.so -- argument marshalling only.

Function names and arguments mirror include/sparq.h.  Tensors are torch CUDA
(ROCm) tensors used purely as device buffers; every step of the computation
runs inside the library's HIP kernels.  There is no CPU fallback: if the
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SPARQ_LIBRARY points at another build of the same library (A/B comparisons); default: the in-tree build
LIB_PATH = os.environ.get("SPARQ_LIBRARY") or os.path.join(_HERE, "libsparq.so")

SPARQ_OK, SPARQ_EINVAL, SPARQ_EUNSUPPORTED, SPARQ_EWORKSPACE, SPARQ_ELAUNCH = range(5)


class SparqMode(ctypes.Structure):
    _fields_ = [("window_bits", ctypes.c_int32), ("shift_mask", ctypes.c_uint32),
                ("round_nearest", ctypes.c_int32), ("pair", ctypes.c_int32)]


class SparqConvDesc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in
                ("B", "H", "W", "C", "N", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w")]


class SparqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    pm, pd = ctypes.POINTER(SparqMode), ctypes.POINTER(SparqConvDesc)
    L.sparq_trim.argtypes = [vp, vp, i64, i32, pm, vp]
    L.sparq_trim.restype = ctypes.c_int
    L.sparq_packed_bytes.argtypes = [pd]
    L.sparq_packed_bytes.restype = sz
    L.sparq_pack_weights.argtypes = [vp, pd, vp, sz, vp]
    L.sparq_pack_weights.restype = ctypes.c_int
    L.sparq_workspace_bytes.argtypes = [pd, pm]
    L.sparq_workspace_bytes.restype = sz
    L.sparq_conv_plan.argtypes = [pd, pm, ctypes.c_char_p, sz]
    L.sparq_conv_plan.restype = ctypes.c_int
    L.sparq_sparse24_plan.argtypes = [pd, pm, ctypes.c_char_p, sz]
    L.sparq_sparse24_plan.restype = ctypes.c_int
    L.sparq_conv_gemm.argtypes = [vp, vp, pd, pm, vp, vp, vp, vp, sz, vp]
    L.sparq_conv_gemm.restype = ctypes.c_int
    L.sparq_conv_gemm_static_ws.argtypes = [vp, vp, pd, pm, vp, vp, vp, vp]
    L.sparq_conv_gemm_static_ws.restype = ctypes.c_int
    L.sparq_dequant.argtypes = [vp, vp, vp, i64, i32, vp]
    L.sparq_dequant.restype = ctypes.c_int
    L.sparq_conv_gemm_u8.argtypes = [vp, vp, pd, pm, vp, vp, pm, vp, sz, vp]
    L.sparq_conv_gemm_u8.restype = ctypes.c_int
    L.sparq_requant.argtypes = [vp, vp, vp, i64, i32, vp]
    L.sparq_requant.restype = ctypes.c_int
    L.sparq_packed_act_bytes.argtypes = [i64, i32, pm, i32]
    L.sparq_packed_act_bytes.restype = sz
    L.sparq_pack_act.argtypes = [vp, vp, sz, i64, i32, pm, i32, vp]
    L.sparq_pack_act.restype = ctypes.c_int
    L.sparq_unpack_act.argtypes = [vp, sz, vp, i64, i32, pm, i32, vp]
    L.sparq_unpack_act.restype = ctypes.c_int
    L.sparq_conv_packed_workspace_bytes.argtypes = [pd, pm]
    L.sparq_conv_packed_workspace_bytes.restype = sz
    L.sparq_conv_gemm_packed.argtypes = [vp, sz, i32, vp, pd, pm, vp, vp, vp, vp, sz, vp]
    L.sparq_conv_gemm_packed.restype = ctypes.c_int
    L.sparq_sparse24_packed_bytes.argtypes = [pd, pm]
    L.sparq_sparse24_packed_bytes.restype = sz
    L.sparq_pack_weights_sparse24.argtypes = [vp, vp, pd, pm, vp, sz, vp]
    L.sparq_pack_weights_sparse24.restype = ctypes.c_int
    L.sparq_sparse24_workspace_bytes.argtypes = [pd, pm]
    L.sparq_sparse24_workspace_bytes.restype = sz
    L.sparq_conv_gemm_sparse24.argtypes = [vp, vp, pd, pm, vp, vp, vp, vp, sz, vp]
    L.sparq_conv_gemm_sparse24.restype = ctypes.c_int
    L.sparq_set_tuning.argtypes = [ctypes.c_char_p]
    L.sparq_set_tuning.restype = ctypes.c_int
    L.sparq_strerror.argtypes = [ctypes.c_int]
    L.sparq_strerror.restype = ctypes.c_char_p
    return L


lib = _load()


def strerror(status: int) -> str:
    return lib.sparq_strerror(int(status)).decode()


def mode(window_bits: int = 4, shift_mask: int = 0x1F, round_nearest: int = 0, pair: int = 1) -> SparqMode:
    return SparqMode(int(window_bits), int(shift_mask), int(round_nearest), int(pair))


def conv_desc(B, H, W, C, N, KH=1, KW=1, stride=(1, 1), pad=(0, 0)) -> SparqConvDesc:
    return SparqConvDesc(B, H, W, C, N, KH, KW, stride[0], stride[1], pad[0], pad[1])


def out_rows(d: SparqConvDesc) -> int:
    Ho = (d.H + 2 * d.pad_h - d.KH) // d.stride_h + 1
    Wo = (d.W + 2 * d.pad_w - d.KW) // d.stride_w + 1
    return d.B * Ho * Wo


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: Optional[torch.Tensor], dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous device tensor of dtype {dtype}")
    return t.data_ptr()


def _check(status: int, what: str) -> None:
    if status != SPARQ_OK:
        raise SparqError(status, what)


def sparq_trim(x: torch.Tensor, y: torch.Tensor, m: SparqMode) -> None:
    """y = vSPARQ/bSPARQ-trimmed x along the last axis (uint8 device tensors; y may be x)."""
    C = x.shape[-1]
    rows = x.numel() // C if C else 0
    if y.shape != x.shape:
        raise ValueError("x and y must have the same shape")
    _check(lib.sparq_trim(_dev(x, torch.uint8, "x"), _dev(y, torch.uint8, "y"), rows, C, ctypes.byref(m), _stream()),
           "sparq_trim")


def sparq_packed_bytes(d: SparqConvDesc) -> int:
    return int(lib.sparq_packed_bytes(ctypes.byref(d)))


def sparq_workspace_bytes(d: SparqConvDesc, m: SparqMode) -> int:
    return int(lib.sparq_workspace_bytes(ctypes.byref(d), ctypes.byref(m)))


def sparq_conv_plan(d: SparqConvDesc, m: SparqMode) -> str:
    """Which kernel and tiling sparq_conv_gemm would use (a line of text for logs)."""
    buf = ctypes.create_string_buffer(256)
    _check(lib.sparq_conv_plan(ctypes.byref(d), ctypes.byref(m), buf, len(buf)), "sparq_conv_plan")
    return buf.value.decode()


def sparq_sparse24_plan(d: SparqConvDesc, m: SparqMode) -> str:
    """Which kernel sparq_conv_gemm_sparse24 would use, and on which matrix instruction (a line of text for logs)."""
    buf = ctypes.create_string_buffer(256)
    _check(lib.sparq_sparse24_plan(ctypes.byref(d), ctypes.byref(m), buf, len(buf)), "sparq_sparse24_plan")
    return buf.value.decode()


def sparq_pack_weights(w: torch.Tensor, d: SparqConvDesc, packed: torch.Tensor) -> None:
    """w int8 [N,KH,KW,C] -> packed (uint8 device buffer of sparq_packed_bytes(d))."""
    if tuple(w.shape) != (d.N, d.KH, d.KW, d.C):
        raise ValueError("weight shape does not match the descriptor")
    _check(lib.sparq_pack_weights(_dev(w, torch.int8, "w"), ctypes.byref(d), _dev(packed, torch.uint8, "packed"),
                                  packed.numel(), _stream()), "sparq_pack_weights")


def sparq_conv_gemm(x: torch.Tensor, packed: torch.Tensor, d: SparqConvDesc, m: SparqMode,
                    acc: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                    out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    if x.numel() != d.B * d.H * d.W * d.C:
        raise ValueError("activation size does not match the descriptor")
    M = out_rows(d)
    for t, nm in ((acc, "acc"), (out, "out")):
        if t is not None and t.numel() != M * d.N:
            raise ValueError(f"{nm} must hold M*N = {M * d.N} elements")
    if scale is not None and scale.numel() != d.N:
        raise ValueError("scale must hold N elements")
    ws_ptr = _dev(workspace, torch.uint8, "workspace")
    ws_bytes = workspace.numel() if workspace is not None else 0
    _check(lib.sparq_conv_gemm(_dev(x, torch.uint8, "x"), _dev(packed, torch.uint8, "packed"), ctypes.byref(d),
                               ctypes.byref(m), _dev(acc, torch.int32, "acc"), _dev(scale, torch.float32, "scale"),
                               _dev(out, torch.float32, "out"), ws_ptr, ws_bytes, _stream()), "sparq_conv_gemm")


def sparq_conv_gemm_static_ws(x: torch.Tensor, packed: torch.Tensor, d: SparqConvDesc, m: SparqMode,
                              acc: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                              out: Optional[torch.Tensor] = None) -> None:
    """sparq_conv_gemm with its scratch taken from the library's own per-GPU array (nothing is allocated)."""
    if x.numel() != d.B * d.H * d.W * d.C:
        raise ValueError("activation size does not match the descriptor")
    M = out_rows(d)
    for t, nm in ((acc, "acc"), (out, "out")):
        if t is not None and t.numel() != M * d.N:
            raise ValueError(f"{nm} must hold M*N = {M * d.N} elements")
    if scale is not None and scale.numel() != d.N:
        raise ValueError("scale must hold N elements")
    _check(lib.sparq_conv_gemm_static_ws(_dev(x, torch.uint8, "x"), _dev(packed, torch.uint8, "packed"), ctypes.byref(d),
                                         ctypes.byref(m), _dev(acc, torch.int32, "acc"),
                                         _dev(scale, torch.float32, "scale"), _dev(out, torch.float32, "out"), _stream()),
           "sparq_conv_gemm_static_ws")


def sparq_dequant(acc: torch.Tensor, scale: torch.Tensor, out: torch.Tensor) -> None:
    M, N = acc.shape
    if out.shape != acc.shape or scale.numel() != N:
        raise ValueError("shape mismatch")
    _check(lib.sparq_dequant(_dev(acc, torch.int32, "acc"), _dev(scale, torch.float32, "scale"),
                             _dev(out, torch.float32, "out"), M, N, _stream()), "sparq_dequant")


def sparq_conv_gemm_u8(x: torch.Tensor, packed: torch.Tensor, d: SparqConvDesc, m: SparqMode, factor: torch.Tensor,
                       y: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                       out_mode: Optional[SparqMode] = None) -> None:
    """The convolution with its result requantised to uint8 (y holds M*N bytes: the next layer's NHWC input),
    optionally trimmed with out_mode as the next layer would trim it on loading."""
    if x.numel() != d.B * d.H * d.W * d.C:
        raise ValueError("activation size does not match the descriptor")
    if y.numel() != out_rows(d) * d.N:
        raise ValueError(f"y must hold M*N = {out_rows(d) * d.N} elements")
    if factor.numel() != d.N:
        raise ValueError("factor must hold N elements")
    ws_ptr = _dev(workspace, torch.uint8, "workspace")
    ws_bytes = workspace.numel() if workspace is not None else 0
    _check(lib.sparq_conv_gemm_u8(_dev(x, torch.uint8, "x"), _dev(packed, torch.uint8, "packed"), ctypes.byref(d),
                                  ctypes.byref(m), _dev(factor, torch.float32, "factor"), _dev(y, torch.uint8, "y"),
                                  ctypes.byref(out_mode) if out_mode is not None else None,
                                  ws_ptr, ws_bytes, _stream()), "sparq_conv_gemm_u8")


def sparq_requant(acc: torch.Tensor, factor: torch.Tensor, y: torch.Tensor) -> None:
    M, N = acc.shape
    if y.shape != acc.shape or factor.numel() != N:
        raise ValueError("shape mismatch")
    _check(lib.sparq_requant(_dev(acc, torch.int32, "acc"), _dev(factor, torch.float32, "factor"),
                             _dev(y, torch.uint8, "y"), M, N, _stream()), "sparq_requant")


def sparq_packed_act_bytes(rows: int, C: int, m: SparqMode, group: int = 1) -> int:
    """Bytes of the packed form of [rows][C] activations (0: this mode / group has none)."""
    return int(lib.sparq_packed_act_bytes(int(rows), int(C), ctypes.byref(m), int(group)))


def sparq_pack_act(x: torch.Tensor, packed: torch.Tensor, m: SparqMode, group: int = 1) -> None:
    """packed (uint8 device buffer) = the n-bit data + ShiftCtrl + MuxCtrl records of the trimmed x (last axis = channels)."""
    C = x.shape[-1]
    _check(lib.sparq_pack_act(_dev(x, torch.uint8, "x"), _dev(packed, torch.uint8, "packed"), packed.numel(),
                              x.numel() // C, C, ctypes.byref(m), int(group), _stream()), "sparq_pack_act")


def sparq_unpack_act(packed: torch.Tensor, y: torch.Tensor, m: SparqMode, group: int = 1) -> None:
    """y (uint8, last axis = channels) = the values the records encode."""
    C = y.shape[-1]
    _check(lib.sparq_unpack_act(_dev(packed, torch.uint8, "packed"), packed.numel(), _dev(y, torch.uint8, "y"),
                                y.numel() // C, C, ctypes.byref(m), int(group), _stream()), "sparq_unpack_act")


def sparq_conv_packed_workspace_bytes(d: SparqConvDesc, m: SparqMode) -> int:
    return int(lib.sparq_conv_packed_workspace_bytes(ctypes.byref(d), ctypes.byref(m)))


def sparq_conv_gemm_packed(packed_x: torch.Tensor, group: int, packed_w: torch.Tensor, d: SparqConvDesc, m: SparqMode,
                           acc: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                           out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    """sparq_conv_gemm on an input held in packed storage (written by sparq_pack_act with the same mode and group)."""
    M = out_rows(d)
    for t, nm in ((acc, "acc"), (out, "out")):
        if t is not None and t.numel() != M * d.N:
            raise ValueError(f"{nm} must hold M*N = {M * d.N} elements")
    if scale is not None and scale.numel() != d.N:
        raise ValueError("scale must hold N elements")
    ws_ptr = _dev(workspace, torch.uint8, "workspace")
    ws_bytes = workspace.numel() if workspace is not None else 0
    _check(lib.sparq_conv_gemm_packed(_dev(packed_x, torch.uint8, "packed_x"), packed_x.numel(), int(group),
                                      _dev(packed_w, torch.uint8, "packed_w"), ctypes.byref(d), ctypes.byref(m),
                                      _dev(acc, torch.int32, "acc"), _dev(scale, torch.float32, "scale"),
                                      _dev(out, torch.float32, "out"), ws_ptr, ws_bytes, _stream()), "sparq_conv_gemm_packed")


def sparq_sparse24_packed_bytes(d: SparqConvDesc, m: SparqMode) -> int:
    return int(lib.sparq_sparse24_packed_bytes(ctypes.byref(d), ctypes.byref(m)))


def sparq_sparse24_workspace_bytes(d: SparqConvDesc, m: SparqMode) -> int:
    return int(lib.sparq_sparse24_workspace_bytes(ctypes.byref(d), ctypes.byref(m)))


def sparq_pack_weights_sparse24(w_vals: torch.Tensor, w_idx: torch.Tensor, d: SparqConvDesc, m: SparqMode,
                                packed: torch.Tensor) -> None:
    """2:4 compressed weights (values int8 and coordinates uint8, both [N,KH,KW,C/2]) -> packed device buffer."""
    if tuple(w_vals.shape) != (d.N, d.KH, d.KW, d.C // 2) or w_idx.shape != w_vals.shape:
        raise ValueError("weight shapes do not match the descriptor")
    _check(lib.sparq_pack_weights_sparse24(_dev(w_vals, torch.int8, "w_vals"), _dev(w_idx, torch.uint8, "w_idx"),
                                           ctypes.byref(d), ctypes.byref(m), _dev(packed, torch.uint8, "packed"),
                                           packed.numel(), _stream()), "sparq_pack_weights_sparse24")


def sparq_conv_gemm_sparse24(x: torch.Tensor, packed: torch.Tensor, d: SparqConvDesc, m: SparqMode,
                             acc: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                             out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    """The convolution with 2:4 pruned weights: activations picked by the weights' coordinates, then paired."""
    if x.numel() != d.B * d.H * d.W * d.C:
        raise ValueError("activation size does not match the descriptor")
    M = out_rows(d)
    for t, nm in ((acc, "acc"), (out, "out")):
        if t is not None and t.numel() != M * d.N:
            raise ValueError(f"{nm} must hold M*N = {M * d.N} elements")
    ws_ptr = _dev(workspace, torch.uint8, "workspace")
    ws_bytes = workspace.numel() if workspace is not None else 0
    _check(lib.sparq_conv_gemm_sparse24(_dev(x, torch.uint8, "x"), _dev(packed, torch.uint8, "packed"), ctypes.byref(d),
                                        ctypes.byref(m), _dev(acc, torch.int32, "acc"), _dev(scale, torch.float32, "scale"),
                                        _dev(out, torch.float32, "out"), ws_ptr, ws_bytes, _stream()), "sparq_conv_gemm_sparse24")


def sparq_set_tuning(spec: Optional[str] = None) -> None:
    """Test / tuning hook: force the kernel choice ("path=patch,patch_tn=128,patch_ws=1", ...); None clears it."""
    _check(lib.sparq_set_tuning(spec.encode() if spec else None), "sparq_set_tuning")
