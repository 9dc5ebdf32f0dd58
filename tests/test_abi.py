"""The C-ABI library loads without a GPU, exports what include/sparq.h declares, and validates
its arguments on the host before touching the device (CPU only: no kernel is launched here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2105_11010_amd", "libsparq.so")
HEADER = os.path.join(ROOT, "include", "sparq.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sparq_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_boundary():
    assert declared_symbols() == ["sparq_conv_gemm", "sparq_conv_gemm_packed", "sparq_conv_gemm_sparse24", "sparq_conv_gemm_static_ws", "sparq_conv_gemm_u8",
                                  "sparq_conv_packed_workspace_bytes", "sparq_conv_plan", "sparq_dequant", "sparq_pack_act",
                                  "sparq_pack_weights", "sparq_pack_weights_sparse24", "sparq_packed_act_bytes", "sparq_packed_bytes", "sparq_requant", "sparq_set_tuning",
                                  "sparq_sparse24_packed_bytes", "sparq_sparse24_plan", "sparq_sparse24_workspace_bytes",
                                  "sparq_strerror", "sparq_trim", "sparq_unpack_act", "sparq_workspace_bytes"]


def test_probe_library_exports_what_its_header_declares():
    """The machine-ceiling micro-benchmarks (a library of their own): loads without a GPU, exports every declared call."""
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "sparq_probe.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(sparq_probe_[a-z0-9_]+)\s*\(", text)))
    assert names == ["sparq_probe_copy", "sparq_probe_mfma_i8", "sparq_probe_mfma_i8_ops"]
    path = os.path.join(ROOT, "paper_2105_11010_amd", "libsparq_probe.so")
    if not os.path.exists(path):
        import __graft_entry__
        __graft_entry__.build()
    L = ctypes.CDLL(path)
    for n in names:
        assert hasattr(L, n), n
    L.sparq_probe_mfma_i8_ops.restype = ctypes.c_double
    L.sparq_probe_mfma_i8_ops.argtypes = [ctypes.c_int32]
    assert L.sparq_probe_mfma_i8_ops(1) == 2.0 * 32768 * 16 * 4 * 256
    assert L.sparq_probe_mfma_i8(None, None, 1, None) == 1          # argument errors come back as codes, nothing is launched
    assert L.sparq_probe_copy(None, None, 16, None) == 1


def test_every_declared_symbol_is_exported(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_binding_matches_header(lib):
    import paper_2105_11010_amd as sq
    for name in declared_symbols():
        assert hasattr(sq, name) or name in ("sparq_strerror",), name
    assert sq.strerror(0) == "ok"
    assert "invalid" in sq.strerror(1)
    assert sq.strerror(99) == "unknown status"


class Mode(ctypes.Structure):
    _fields_ = [("window_bits", ctypes.c_int32), ("shift_mask", ctypes.c_uint32),
                ("round_nearest", ctypes.c_int32), ("pair", ctypes.c_int32)]


class Desc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in
                ("B", "H", "W", "C", "N", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w")]


def test_layout_queries(lib):
    lib.sparq_packed_bytes.restype = ctypes.c_size_t
    lib.sparq_workspace_bytes.restype = ctypes.c_size_t
    d = Desc(1, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1)
    m = Mode(4, 0x1F, 1, 1)
    # N padded to 256, K = 576 padded to 576 (multiple of 64): 256*4 colsum bytes + 576*256 weight bytes
    assert lib.sparq_packed_bytes(ctypes.byref(d)) == 256 * 4 + 576 * 256
    assert lib.sparq_workspace_bytes(ctypes.byref(d), ctypes.byref(m)) == 0      # 25 tiles x 1 channel block: nothing to split
    # 65 channels: a channel-padded (80) copy of x, 256-byte granular; a layer this small may also be
    # given room for the int32 partial sums of a split reduction (100 x 12 outputs)
    d_odd = Desc(1, 10, 10, 65, 12, 3, 3, 1, 1, 1, 1)
    pad = 100 * 80 + (256 - (100 * 80) % 256) % 256
    assert lib.sparq_workspace_bytes(ctypes.byref(d_odd), ctypes.byref(m)) in (pad, pad + 100 * 12 * 4 + (256 - (100 * 12 * 4) % 256) % 256)
    bad = Desc(1, 2, 2, 64, 64, 3, 3, 1, 1, 0, 0)       # kernel larger than the image
    assert lib.sparq_packed_bytes(ctypes.byref(bad)) == 0
    assert lib.sparq_packed_bytes(None) == 0
    huge_k = Desc(1, 1, 1, 70000, 8, 1, 1, 1, 1, 0, 0)  # 255*127*K leaves int32
    assert lib.sparq_packed_bytes(ctypes.byref(huge_k)) == 0


def test_argument_validation_returns_codes(lib):
    EINVAL = 1
    m = Mode(4, 0x1F, 1, 1)
    d = Desc(1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 1)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    assert lib.sparq_trim(None, fake, 1, 16, ctypes.byref(m), None) == EINVAL
    assert lib.sparq_trim(fake, fake, ctypes.c_int64(-1), 16, ctypes.byref(m), None) == EINVAL
    assert lib.sparq_trim(fake, fake, ctypes.c_int64(1), 0, ctypes.byref(m), None) == EINVAL
    for bad in (Mode(4, 0x0F, 0, 1), Mode(4, 0x1E, 0, 1), Mode(5, 0x1F, 0, 1), Mode(4, 0x3F, 0, 0),
                Mode(4, 0x1F, 2, 1), Mode(2, 0x41, 0, 1), Mode(3, 0x2B, 0, 1)):
        assert lib.sparq_trim(fake, fake, ctypes.c_int64(1), 16, ctypes.byref(bad), None) == EINVAL
    assert lib.sparq_trim(fake, fake, ctypes.c_int64(1), 16, None, None) == EINVAL
    # partial overlap of x and y
    assert lib.sparq_trim(ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008), ctypes.c_int64(1), 16,
                          ctypes.byref(m), None) == EINVAL
    assert lib.sparq_trim(fake, fake, ctypes.c_int64(0), 16, ctypes.byref(m), None) == 0     # empty: nothing to do
    assert lib.sparq_dequant(None, fake, fake, ctypes.c_int64(1), 4, None) == EINVAL
    assert lib.sparq_dequant(fake, fake, fake, ctypes.c_int64(1), 0, None) == EINVAL
    assert lib.sparq_requant(None, fake, fake, ctypes.c_int64(1), 4, None) == EINVAL
    assert lib.sparq_requant(fake, fake, fake, ctypes.c_int64(-1), 4, None) == EINVAL
    assert lib.sparq_requant(fake, fake, fake, ctypes.c_int64(0), 4, None) == 0
    assert lib.sparq_dequant(fake, fake, fake, ctypes.c_int64(0), 4, None) == 0
    assert lib.sparq_pack_weights(None, ctypes.byref(d), fake, ctypes.c_size_t(1 << 20), None) == EINVAL
    assert lib.sparq_pack_weights(fake, ctypes.byref(d), ctypes.c_void_p(0x1010), ctypes.c_size_t(1 << 20), None) == EINVAL
    assert lib.sparq_pack_weights(fake, ctypes.byref(d), fake, ctypes.c_size_t(16), None) == 3   # buffer too small
    args = (fake, fake, ctypes.byref(d), ctypes.byref(m))
    assert lib.sparq_conv_gemm(*args, None, None, None, None, ctypes.c_size_t(0), None) == EINVAL       # no output
    assert lib.sparq_conv_gemm(*args, None, None, fake, None, ctypes.c_size_t(0), None) == EINVAL       # out without scale
    assert lib.sparq_conv_gemm(None, fake, ctypes.byref(d), ctypes.byref(m), fake, None, None, None,
                               ctypes.c_size_t(0), None) == EINVAL
    assert lib.sparq_conv_gemm(ctypes.c_void_p(0x1004), fake, ctypes.byref(d), ctypes.byref(m), fake, None, None,
                               None, ctypes.c_size_t(0), None) == EINVAL                               # misaligned x
    d_odd = Desc(1, 10, 10, 65, 12, 3, 3, 1, 1, 1, 1)
    assert lib.sparq_conv_gemm(fake, fake, ctypes.byref(d_odd), ctypes.byref(m), fake, None, None, None,
                               ctypes.c_size_t(0), None) == EINVAL                                     # workspace missing
    assert lib.sparq_conv_gemm(fake, fake, ctypes.byref(d_odd), ctypes.byref(m), fake, None, None, fake,
                               ctypes.c_size_t(16), None) == 3                                         # workspace too small
    # the requantised-output entry point: factor and y are both required, y aligned, out_mode valid if given
    u8 = (fake, fake, ctypes.byref(d), ctypes.byref(m))
    assert lib.sparq_conv_gemm_u8(*u8, None, fake, None, None, ctypes.c_size_t(0), None) == EINVAL      # no factor
    assert lib.sparq_conv_gemm_u8(*u8, fake, None, None, None, ctypes.c_size_t(0), None) == EINVAL      # no y
    assert lib.sparq_conv_gemm_u8(*u8, fake, ctypes.c_void_p(0x1004), None, None, ctypes.c_size_t(0), None) == EINVAL
    bad = Mode(4, 0x0F, 0, 1)
    assert lib.sparq_conv_gemm_u8(*u8, fake, fake, ctypes.byref(bad), None, ctypes.c_size_t(0), None) == EINVAL
    assert lib.sparq_conv_gemm_u8(fake, fake, ctypes.byref(d_odd), ctypes.byref(m), fake, fake, None, None,
                                  ctypes.c_size_t(0), None) == EINVAL                                  # workspace missing

