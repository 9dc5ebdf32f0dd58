"""Host-side planning of the convolution (no GPU): every layer of the workload tables gets a plan,
and the plan agrees with the workspace the library asks for."""
import ctypes
import os

import pytest

import sparq_synth as S

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(os.path.dirname(HERE), "paper_2105_11010_amd", "libsparq.so")


class Mode(ctypes.Structure):
    _fields_ = [("window_bits", ctypes.c_int32), ("shift_mask", ctypes.c_uint32),
                ("round_nearest", ctypes.c_int32), ("pair", ctypes.c_int32)]


class Desc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in
                ("B", "H", "W", "C", "N", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w")]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.skip("libsparq.so not built")
    L = ctypes.CDLL(LIB)
    L.sparq_workspace_bytes.restype = ctypes.c_size_t
    L.sparq_packed_bytes.restype = ctypes.c_size_t
    return L


def plan(lib, l, mode=None):
    d = Desc(l.B, l.H, l.W, l.C, l.N, l.KH, l.KW, l.stride[0], l.stride[1], l.pad[0], l.pad[1])
    m = Mode(*(mode or l.mode).astuple())
    buf = ctypes.create_string_buffer(256)
    assert lib.sparq_conv_plan(ctypes.byref(d), ctypes.byref(m), buf, len(buf)) == 0
    return buf.value.decode(), lib.sparq_workspace_bytes(ctypes.byref(d), ctypes.byref(m)), lib.sparq_packed_bytes(ctypes.byref(d))


ALL = [(c, l) for c, ls in ((0, S.config0()), (1, S.config1()), (2, S.config2()), (4, S.config4())) for l in ls]


@pytest.mark.parametrize("cfg,layer", ALL, ids=lambda v: v.name if hasattr(v, "name") else f"cfg{v}")
def test_every_workload_layer_has_a_consistent_plan(lib, cfg, layer):
    text, ws, packed = plan(lib, layer)
    assert text.startswith(("conv_patch_kernel", "conv_gemm_kernel"))
    pixels = layer.B * layer.H * layer.W
    if layer.C <= 4:
        assert "pixel_folded" in text and ws >= pixels * 4           # 4-channel padded copy
    elif layer.C % 16:
        assert "padded_copy" in text and ws >= pixels * ((layer.C + 15) // 16 * 16)
    else:
        assert "padded_copy" not in text
    if layer.C % 16 == 0:
        assert ws == 0                                                # nothing to stage
    assert packed >= layer.K * layer.N


def test_plan_of_the_headline_shapes(lib):
    conv = S.ConvLayer("conv3x3", 64, 32, 32, 512, 512, 3, 3, (1, 1), (1, 1), 0.5, S.Mode(4, S.OPT5, 1, 1))
    text, ws, _ = plan(lib, conv)
    assert text.startswith("conv_patch_kernel tile=128x256") and "wave_specialised" in text and ws == 0
    text, ws, _ = plan(lib, S.config3_layer())
    assert text.startswith("conv_gemm_kernel tile=128x512") and ws == 0


def test_tuning_hook_forces_and_clears_the_choice(lib):
    """sparq_set_tuning: the documented keys change the plan, NULL restores the rules, junk is refused and changes nothing."""
    conv = S.ConvLayer("conv3x3", 64, 32, 32, 512, 512, 3, 3, (1, 1), (1, 1), 0.5, S.Mode(4, S.OPT5, 1, 1))
    lib.sparq_set_tuning.argtypes = [ctypes.c_char_p]
    base = plan(lib, conv)[0]
    try:
        assert lib.sparq_set_tuning(b"path=gather,tile=128x256") == 0
        assert plan(lib, conv)[0].startswith("conv_gemm_kernel tile=128x256")
        assert lib.sparq_set_tuning(b"path=patch,patch_tn=64,patch_ws=0") == 0
        text = plan(lib, conv)[0]
        assert text.startswith("conv_patch_kernel tile=128x64") and "wave_specialised" not in text
        for junk in (b"path=fast", b"tile=64x64", b"patch_tn=100", b"patch_ws=2", b"colour=red", b"path", b","):
            assert lib.sparq_set_tuning(junk) == 1
        assert plan(lib, conv)[0] == text                            # a refused spec leaves the override as it was
    finally:
        assert lib.sparq_set_tuning(None) == 0
    assert plan(lib, conv)[0] == base


def test_widest_gather_tile_only_with_step_aligned_taps(lib):
    """The 128 x 512 tile tracks a step's filter tap in scalar registers, so every 64-byte reduction step must lie
    inside one tap (more than 32 channels); otherwise, and when 512 columns would read past the padded weights, the
    library takes the next tile, also when the hook asks for the widest one."""
    lib.sparq_set_tuning.argtypes = [ctypes.c_char_p]
    mode = S.Mode(4, S.OPT5, 1, 1)
    try:
        assert lib.sparq_set_tuning(b"path=gather,tile=128x512") == 0
        assert plan(lib, S.ConvLayer("c64", 1, 9, 9, 64, 300, 3, 3, (1, 1), (1, 1)), mode)[0].startswith("conv_gemm_kernel tile=128x512")
        assert plan(lib, S.ConvLayer("c32", 1, 9, 9, 32, 300, 3, 3, (1, 1), (1, 1)), mode)[0].startswith("conv_gemm_kernel tile=128x256")
        assert plan(lib, S.ConvLayer("n520", 1, 9, 9, 64, 520, 3, 3, (1, 1), (1, 1)), mode)[0].startswith("conv_gemm_kernel tile=128x256")
    finally:
        assert lib.sparq_set_tuning(None) == 0


def test_plan_rejects_bad_arguments(lib):
    buf = ctypes.create_string_buffer(64)
    m = Mode(4, 0x1F, 1, 1)
    bad = Desc(1, 2, 2, 64, 64, 3, 3, 1, 1, 0, 0)
    assert lib.sparq_conv_plan(ctypes.byref(bad), ctypes.byref(m), buf, len(buf)) == 1
    ok = Desc(1, 8, 8, 64, 64, 3, 3, 1, 1, 1, 1)
    assert lib.sparq_conv_plan(ctypes.byref(ok), ctypes.byref(m), None, 0) == 1
    assert lib.sparq_conv_plan(ctypes.byref(ok), ctypes.byref(Mode(5, 1, 0, 0)), buf, len(buf)) == 1


def sparse_plan(lib, d, m):
    buf = ctypes.create_string_buffer(256)
    assert lib.sparq_sparse24_plan(ctypes.byref(d), ctypes.byref(m), buf, len(buf)) == 0
    return buf.value.decode()


def test_sparse24_plan_names_the_matrix_instruction(lib):
    """2:4 pruned weights: the sparse matrix instruction wherever the (expanded) layer takes the wave-specialised
    input-patch kernel, for every mode; the dense kernels where it does not; and the packed buffer holds both forms."""
    lib.sparq_sparse24_packed_bytes.restype = ctypes.c_size_t
    conv = Desc(64, 32, 32, 512, 512, 3, 3, 1, 1, 1, 1)
    for m in (Mode(4, 0x1F, 1, 1), Mode(4, 0x1F, 1, 0), Mode(4, 0x15, 0, 0), Mode(3, 0x3F, 1, 0), Mode(8, 1, 0, 0)):
        text = sparse_plan(lib, conv, m)
        assert text.startswith("conv_patch_kernel tile=128x256") and text.endswith("sparse_mfma"), text
        assert ("expanded_x4" in text) == bool(m.pair and m.window_bits != 8), text
    thin = Desc(2, 8, 8, 4, 8, 1, 1, 1, 1, 0, 0)                      # expands to 16 channels: taps are not step-aligned
    assert sparse_plan(lib, thin, Mode(4, 0x1F, 1, 1)).endswith("dense_mfma")
    assert lib.sparq_set_tuning(b"path=gather") == 0
    try:
        assert sparse_plan(lib, conv, Mode(4, 0x1F, 1, 1)).endswith("dense_mfma")
    finally:
        assert lib.sparq_set_tuning(None) == 0
    m = Mode(4, 0x1F, 1, 1)
    lib.sparq_packed_bytes.restype = ctypes.c_size_t
    eff = Desc(64, 32, 32, 2048, 512, 3, 3, 1, 1, 1, 1)
    dense_tiles = lib.sparq_packed_bytes(ctypes.byref(eff))
    kp_np = 9 * 2048 * 512
    assert lib.sparq_sparse24_packed_bytes(ctypes.byref(conv), ctypes.byref(m)) >= dense_tiles + kp_np + kp_np // 2 + kp_np // 8
    buf = ctypes.create_string_buffer(64)
    assert lib.sparq_sparse24_plan(ctypes.byref(Desc(1, 4, 4, 6, 8, 1, 1, 1, 1, 0, 0)), ctypes.byref(m), buf, len(buf)) == 1   # C % 4
