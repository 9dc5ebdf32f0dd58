"""GPU parity: libsparq (HIP, through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import sparq_synth as S

pytestmark = pytest.mark.gpu

MODES_N4 = [S.Mode(4, m, r, p) for m in (S.OPT5, S.OPT3, S.OPT2) for r in (0, 1) for p in (0, 1)]
MODES_LOW = [S.Mode(2, S.OPT7_2B, r, p) for r in (0, 1) for p in (0, 1)] + \
            [S.Mode(3, S.OPT6_3B, r, p) for r in (0, 1) for p in (0, 1)]
MODES_ODD = [S.Mode(4, 0x1B, 1, 1), S.Mode(4, 0x13, 0, 1), S.Mode(3, 0x2D, 1, 1), S.Mode(2, 0x5F, 1, 1), S.PLAIN8]


@pytest.fixture(scope="module")
def sq():
    assert torch.cuda.is_available(), "GPU tests need a device"
    import paper_2105_11010_amd as sq_
    return sq_


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def run_conv(sq, x, w, sc, layer, mode, want_acc=True, want_out=True):
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    m = sq.mode(*mode.astuple())
    xd, wd, sd = dev(x), dev(w), dev(sc)
    packed = torch.empty(sq.sparq_packed_bytes(d), dtype=torch.uint8, device="cuda:0")
    sq.sparq_pack_weights(wd, d, packed)
    wsb = sq.sparq_workspace_bytes(d, m)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda:0") if wsb else None
    acc = torch.full((layer.M, layer.N), -7, dtype=torch.int32, device="cuda:0") if want_acc else None
    out = torch.full((layer.M, layer.N), -7.0, dtype=torch.float32, device="cuda:0") if want_out else None
    sq.sparq_conv_gemm(xd, packed, d, m, acc=acc, scale=sd if want_out else None, out=out, workspace=ws)
    torch.cuda.synchronize()
    return (acc.cpu().numpy() if want_acc else None), (out.cpu().numpy() if want_out else None)


def check_layer(sq, oracle, layer, mode, seed_cfg=8, rows=None):
    x, w, sc = S.gen_layer(seed_cfg, layer)
    acc, out = run_conv(sq, x, w, sc, layer, mode)
    ref_acc, ref_out = oracle.conv_gemm(x, w, layer.stride, layer.pad, scale=sc, rows=rows, **mode.kwargs())
    if rows is not None:
        acc, out = acc[rows], out[rows]
    assert np.array_equal(acc, ref_acc), f"{layer.name} {mode.label}: int32 mismatch"
    # fp32 dequantised output within 1e-6 relative of the fp64 oracle
    err = np.abs(out.astype(np.float64) - ref_out)
    assert np.all(err <= 1e-6 * np.abs(ref_out)), f"{layer.name} {mode.label}: fp32 output off"


# ---------------------------------------------------------------- trim ------

@pytest.mark.parametrize("mode", MODES_N4 + MODES_LOW + MODES_ODD, ids=lambda m: m.label + f"-{m.shift_mask:#x}")
def test_trim_all_pairs(sq, oracle, mode):
    """All 256 x 256 activation pairs, in both byte lanes of the packed word."""
    a, b = np.meshgrid(np.arange(256, dtype=np.uint8), np.arange(256, dtype=np.uint8), indexing="ij")
    x = np.stack([a, b, b, a], axis=-1).reshape(-1, 4)
    xd = dev(x)
    y = torch.empty_like(xd)
    sq.sparq_trim(xd, y, sq.mode(*mode.astuple()))
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), oracle.trim(x, **mode.kwargs()))


@pytest.mark.parametrize("C", [1, 2, 3, 6, 7, 16, 30, 33, 64, 159])
@pytest.mark.parametrize("mode", [S.Mode(4, S.OPT5, 1, 1), S.Mode(4, S.OPT3, 0, 1), S.Mode(2, S.OPT7_2B, 1, 1)],
                         ids=lambda m: m.label)
def test_trim_row_lengths(sq, oracle, C, mode):
    """Odd and ragged channel counts: the last channel of an odd row has no partner."""
    rng = S.rng_for(8, 100 + C)
    for rows in (1, 5, 1031):
        x = S.gen_activations((rows, C), 0.5, rng)
        xd = dev(x)
        y = torch.empty_like(xd)
        sq.sparq_trim(xd, y, sq.mode(*mode.astuple()))
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), oracle.trim(x, **mode.kwargs())), (rows, C)


def test_trim_in_place_large_and_empty(sq, oracle):
    mode = S.Mode(4, S.OPT5, 1, 1)
    x = S.gen_activations((4099, 96), 0.5, S.rng_for(8, 200))
    xd = dev(x)
    sq.sparq_trim(xd, xd, sq.mode(*mode.astuple()))
    torch.cuda.synchronize()
    assert np.array_equal(xd.cpu().numpy(), oracle.trim(x, **mode.kwargs()))
    e = torch.empty((0, 8), dtype=torch.uint8, device="cuda:0")
    sq.sparq_trim(e, e, sq.mode(*mode.astuple()))


def test_trim_streamed_form(sq, oracle):
    """A call that moves 256 MiB or more out of place takes the kernel with non-temporal accesses: every byte
    against the oracle on a 136 MB tensor with a ragged tail (one 16-byte word plus a few pairs left over)."""
    mode = S.Mode(4, S.OPT3, 1, 1)
    block = S.gen_activations((1 << 22,), 0.5, S.rng_for(8, 210))
    x = np.resize(block, (1, (136 << 20) + 22))
    xd, yd = dev(x), torch.zeros(x.shape, dtype=torch.uint8, device="cuda:0")
    sq.sparq_trim(xd, yd, sq.mode(*mode.astuple()))
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy(), oracle.trim(x, **mode.kwargs()))


# ------------------------------------------------------------- dequant ------

@pytest.mark.parametrize("M,N", [(1, 1), (37, 19), (513, 64), (1000, 160)])
def test_dequant(sq, oracle, M, N):
    rng = S.rng_for(8, 300 + N)
    acc = rng.integers(-2 ** 31, 2 ** 31, size=(M, N), dtype=np.int64).astype(np.int32)
    sc = S.gen_scales(N, rng)
    out = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    sq.sparq_dequant(dev(acc), dev(sc), out)
    torch.cuda.synchronize()
    ref = oracle.dequant(acc, sc)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    assert np.all(err <= 1e-6 * np.abs(ref))


def test_dequant_streamed_form(sq, oracle):
    """8 * M * N >= 256 MiB: the dequantisation kernel with non-temporal accesses, every element."""
    M, N = 65537, 512
    rng = S.rng_for(8, 310)
    acc = np.resize(rng.integers(-2 ** 31, 2 ** 31, size=(1 << 20,), dtype=np.int64).astype(np.int32), (M, N))
    sc = S.gen_scales(N, rng)
    out = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    sq.sparq_dequant(dev(acc), dev(sc), out)
    torch.cuda.synchronize()
    ref = oracle.dequant(acc, sc)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    assert np.all(err <= 1e-6 * np.abs(ref))


# ------------------------------------------------------------- requant ------

@pytest.mark.parametrize("M,N", [(1, 1), (37, 19), (513, 64), (1000, 160), (0, 8)])
def test_requant(sq, oracle, M, N):
    """The standalone requantisation pass: bit-exact bytes, ties and both clamps included."""
    rng = S.rng_for(8, 400 + N)
    acc = rng.integers(-60000, 200000, size=(M, N), dtype=np.int64).astype(np.int32)
    if M:
        acc[0, 0] = 5                       # 2.5 with factor 0.5: the tie
    f = rng.uniform(5e-4, 3e-3, size=N).astype(np.float32)
    f[0] = 0.5
    y = torch.full((M, N), 7, dtype=torch.uint8, device="cuda:0")
    sq.sparq_requant(dev(acc), dev(f), y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), oracle.requant(acc, f))


def run_conv_u8(sq, x, w, f, layer, mode, out_mode=None):
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    m = sq.mode(*mode.astuple())
    packed = torch.empty(sq.sparq_packed_bytes(d), dtype=torch.uint8, device="cuda:0")
    sq.sparq_pack_weights(dev(w), d, packed)
    wsb = sq.sparq_workspace_bytes(d, m)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda:0") if wsb else None
    y = torch.full((layer.M, layer.N), 7, dtype=torch.uint8, device="cuda:0")
    sq.sparq_conv_gemm_u8(dev(x), packed, d, m, dev(f), y, workspace=ws,
                          out_mode=sq.mode(*out_mode.astuple()) if out_mode else None)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check_layer_u8(sq, oracle, layer, mode, seed_cfg=8, out_mode=None):
    """Requantised uint8 output of the fused convolution (optionally trimmed for the next layer): every byte
    equals the oracle's."""
    x, w, _ = S.gen_layer(seed_cfg, layer)
    f = S.gen_requant(layer, S.rng_for(seed_cfg, 900 + layer.index))
    y = run_conv_u8(sq, x, w, f, layer, mode, out_mode)
    ref = oracle.conv_gemm_u8(x, w, f, layer.stride, layer.pad, out_mode=out_mode.kwargs() if out_mode else None,
                              **mode.kwargs())
    assert np.array_equal(y, ref), f"{layer.name} {mode.label}: uint8 mismatch"
    assert (ref == 0).any() and ref.max() > 60, "degenerate test case"


@pytest.mark.parametrize("N", [4, 3])
def test_requant_every_tie_and_both_clamps(sq, oracle, N):
    """Factors 0.5 and 0.25 over a run of consecutive accumulators: every second / fourth product is a tie;
    negative products clamp to 0, large ones to 255 (N = 4: the vector kernel, N = 3: the scalar one)."""
    acc = np.arange(-600, 600 + 1200 * N, dtype=np.int32)[:1200 * N].reshape(1200, N)
    f = np.array([0.5, 0.25, 0.5, 0.125][:N], dtype=np.float32)
    y = torch.full((1200, N), 7, dtype=torch.uint8, device="cuda:0")
    sq.sparq_requant(dev(acc), dev(f), y)
    torch.cuda.synchronize()
    ref = oracle.requant(acc, f)
    assert np.array_equal(y.cpu().numpy(), ref)
    assert (ref == 0).any() and (ref == 255).any()


# ---------------------------------------------------------- conv / gemm -----

def test_config0_full(sq, oracle):
    (layer,) = S.config0()
    x, w, sc = S.gen_layer(0, layer)
    acc, out = run_conv(sq, x, w, sc, layer, layer.mode)
    ref_acc, ref_out = oracle.conv_gemm(x, w, layer.stride, layer.pad, scale=sc, **layer.mode.kwargs())
    assert np.array_equal(acc, ref_acc)
    assert np.all(np.abs(out.astype(np.float64) - ref_out) <= 1e-6 * np.abs(ref_out))


SHAPES = [
    # name, B, H, W, C, N, KH, KW, stride, pad
    S.ConvLayer("gemm_small", 1, 300, 1, 64, 32),
    S.ConvLayer("gemm_ragged", 1, 777, 1, 208, 100),
    S.ConvLayer("gemm_k16", 1, 130, 1, 16, 8),
    S.ConvLayer("gemm_k48_n3", 1, 129, 1, 48, 3),
    S.ConvLayer("1x1_s2", 3, 15, 13, 32, 40, 1, 1, (2, 2), (0, 0)),
    S.ConvLayer("3x3_p1", 2, 13, 11, 32, 24, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("3x3_s2_p1", 2, 17, 19, 48, 36, 3, 3, (2, 2), (1, 1)),
    S.ConvLayer("3x3_s2_p0", 1, 17, 17, 96, 20, 3, 3, (2, 2), (0, 0)),
    S.ConvLayer("5x5_p2", 1, 12, 12, 48, 64, 5, 5, (1, 1), (2, 2)),
    S.ConvLayer("1x7", 2, 9, 17, 32, 33, 1, 7, (1, 1), (0, 3)),
    S.ConvLayer("7x1", 2, 17, 9, 160, 17, 7, 1, (1, 1), (3, 0)),
    S.ConvLayer("odd_c65", 1, 10, 10, 65, 12, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("odd_c3_7x7", 2, 20, 20, 3, 16, 7, 7, (2, 2), (3, 3)),
    S.ConvLayer("odd_c159_n161", 1, 6, 17, 159, 161, 1, 7, (1, 1), (0, 3)),
    S.ConvLayer("wide_n", 1, 140, 1, 128, 520),
    # at most 4 channels: the pixel-folded first-layer path (and shapes that cannot fold)
    S.ConvLayer("thin_3x3_s1_c3", 2, 9, 16, 3, 10, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("thin_5x5_s2_c4", 1, 12, 24, 4, 7, 5, 5, (2, 2), (2, 2)),
    S.ConvLayer("thin_7x7_s2_c1", 3, 16, 32, 1, 64, 7, 7, (2, 2), (3, 3)),
    S.ConvLayer("thin_3x3_s2_c2_n130", 2, 10, 40, 2, 130, 3, 3, (2, 2), (1, 1)),
    S.ConvLayer("thin_s4_no_fold", 1, 16, 32, 1, 5, 3, 3, (4, 4), (1, 1)),
    S.ConvLayer("thin_w18_no_fold", 1, 7, 18, 3, 9, 3, 3, (1, 1), (1, 1)),
]


# The library holds two convolution kernels (an im2col-gather form and an input-patch form) and
# picks one per layer; the tuning hook (sparq_set_tuning) forces either where the layer is eligible,
# so both are compared with the oracle on every shape.
@pytest.fixture
def tuning(sq):
    """tuning("path=patch,patch_tn=128") forces the kernel choice for the rest of the test."""
    yield sq.sparq_set_tuning
    sq.sparq_set_tuning(None)


@pytest.fixture(params=["auto", "gather", "patch", "patch-ws"])
def path(request, tuning):
    if request.param == "patch-ws":      # the wave-specialised form of the patch kernel
        tuning("path=patch,patch_ws=1")
    elif request.param != "auto":
        tuning(f"path={request.param},patch_ws=0")
    return request.param


@pytest.mark.parametrize("layer", SHAPES, ids=lambda l: l.name)
@pytest.mark.parametrize("mode", [S.Mode(4, S.OPT5, 1, 1), S.Mode(4, S.OPT3, 0, 1), S.Mode(2, S.OPT7_2B, 1, 1), S.PLAIN8],
                         ids=lambda m: m.label)
def test_conv_shapes(sq, oracle, layer, mode, path):
    check_layer(sq, oracle, layer, mode, seed_cfg=8)


# Shapes chosen for the input-patch kernel: tiles that span several image rows and several images,
# one-row tiles, every staging variant (64/128/256-channel units), several output-channel tiles.
PATCH_SHAPES = [
    S.ConvLayer("p_3x3_56_c64_n64", 2, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("p_3x3_8x8_c128_n300", 9, 8, 8, 128, 300, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("p_3x3_7x7_c64_n96", 11, 7, 7, 64, 96, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("p_3x3_wide_row", 1, 5, 300, 64, 40, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("p_5x5_c48", 3, 20, 20, 48, 70, 5, 5, (1, 1), (2, 2)),
    S.ConvLayer("p_1x3_c384", 5, 8, 8, 384, 130, 1, 3, (1, 1), (0, 1)),
    S.ConvLayer("p_3x1_c96", 5, 8, 8, 96, 64, 3, 1, (1, 1), (1, 0)),
    S.ConvLayer("p_1x1_c64", 1, 37, 41, 64, 256),
    S.ConvLayer("p_1x1_c128", 2, 30, 30, 128, 192),
    S.ConvLayer("p_1x1_c256", 1, 50, 27, 256, 72),
    S.ConvLayer("p_1x1_c768", 1, 33, 33, 768, 128),
    S.ConvLayer("p_1x1_c80", 1, 19, 23, 80, 50),
    S.ConvLayer("p_3x3_s2_small", 6, 9, 9, 64, 32, 3, 3, (2, 2), (1, 1)),
    S.ConvLayer("p_3x3_p2_dilated_pad", 2, 6, 6, 64, 16, 3, 3, (1, 1), (2, 2)),
    S.ConvLayer("p_2x2_even_taps", 2, 10, 10, 64, 16, 2, 2, (1, 1), (0, 0)),
    S.ConvLayer("p_1x1_s2_c64_n48", 3, 15, 13, 64, 48, 1, 1, (2, 2), (0, 0)),      # strided 1x1: pixel remap
    S.ConvLayer("p_1x1_s2_c128_n200", 5, 14, 14, 128, 200, 1, 1, (2, 2), (0, 0)),
    S.ConvLayer("p_1x1_s3x2_c256_n70", 2, 17, 19, 256, 70, 1, 1, (3, 2), (0, 0)),
]


@pytest.mark.parametrize("layer", PATCH_SHAPES, ids=lambda l: l.name)
@pytest.mark.parametrize("mode", [S.Mode(4, S.OPT5, 1, 1), S.Mode(3, S.OPT6_3B, 0, 1)], ids=lambda m: m.label)
def test_conv_patch_shapes(sq, oracle, layer, mode, path):
    check_layer(sq, oracle, layer, mode, seed_cfg=9)


@pytest.mark.parametrize("layer", SHAPES + PATCH_SHAPES, ids=lambda l: l.name)
def test_conv_u8_shapes(sq, oracle, layer, path):
    """The requantised-output entry point on every shape and through every kernel form."""
    check_layer_u8(sq, oracle, layer, S.Mode(4, S.OPT5, 1, 1), seed_cfg=9)


@pytest.mark.parametrize("layer", SHAPES + PATCH_SHAPES, ids=lambda l: l.name)
@pytest.mark.parametrize("mode", [S.Mode(4, S.OPT5, 1, 1), S.Mode(3, S.OPT6_3B, 0, 1)], ids=lambda m: m.label)
def test_conv_u8_trimmed_for_the_next_layer(sq, oracle, layer, mode, path):
    """Output trimmed with the layer's own mode: inside the epilogue where N is a multiple of 4, by a pass of the
    standalone trim otherwise (odd N: the last channel of a pixel has no partner)."""
    check_layer_u8(sq, oracle, layer, mode, seed_cfg=9, out_mode=mode)


@pytest.mark.parametrize("layer", SHAPES + PATCH_SHAPES, ids=lambda l: l.name)
def test_conv_u8_untrimmed_input_trimmed_output(sq, oracle, layer, path):
    """The steady state of a chain: the input arrives trimmed (this layer runs at plain 8 bits) and the output is
    trimmed for the next one -- in the wave-specialised kernels' epilogue, by a trim pass in the other forms."""
    check_layer_u8(sq, oracle, layer, S.PLAIN8, seed_cfg=9, out_mode=S.Mode(4, S.OPT5, 1, 1))


@pytest.mark.parametrize("mode,out_mode", [(S.PLAIN8, S.Mode(4, S.OPT5, 1, 1)), (S.Mode(4, S.OPT5, 1, 1), S.Mode(4, S.OPT3, 0, 0)),
                                           (S.Mode(4, S.OPT2, 0, 1), S.PLAIN8)], ids=["plain-to-5opt", "5opt-to-3opt", "2opt-to-plain"])
def test_conv_u8_trimmed_with_another_mode(sq, oracle, mode, out_mode):
    """A first layer at plain 8 bits feeding a trimmed one, two different modes, and no output trim."""
    for layer in (S.ConvLayer("u8_tm_a", 2, 12, 12, 64, 96, 3, 3, (1, 1), (1, 1)), S.ConvLayer("u8_tm_b", 1, 9, 30, 3, 64, 7, 7, (2, 2), (3, 3))):
        check_layer_u8(sq, oracle, layer, mode, seed_cfg=9, out_mode=out_mode)


def test_conv_u8_trimmed_chain_runs_the_second_layer_untrimmed(sq, oracle):
    """Layer 1 trims its output for layer 2; layer 2 at plain 8 bits then equals layer 2 trimming on load."""
    l1 = S.ConvLayer("tchain1", 2, 12, 12, 64, 96, 3, 3, (1, 1), (1, 1))
    l2 = S.ConvLayer("tchain2", 2, 12, 12, 96, 40, 1, 1, index=1)
    mode = S.Mode(4, S.OPT5, 1, 1)
    x, w1, _ = S.gen_layer(9, l1)
    _, w2, _ = S.gen_layer(9, l2)
    f1, f2 = S.gen_requant(l1, S.rng_for(9, 950)), S.gen_requant(l2, S.rng_for(9, 951))
    y1t = run_conv_u8(sq, x, w1, f1, l1, mode, out_mode=mode)
    y2 = run_conv_u8(sq, y1t.reshape(l2.x_shape()), w2, f2, l2, S.PLAIN8)
    r1 = oracle.conv_gemm_u8(x, w1, f1, l1.stride, l1.pad, **mode.kwargs())            # untrimmed bytes
    r2 = oracle.conv_gemm_u8(r1.reshape(l2.x_shape()), w2, f2, l2.stride, l2.pad, **mode.kwargs())   # trimmed on load
    assert np.array_equal(y1t, oracle.trim(r1, **mode.kwargs())) and np.array_equal(y2, r2)


@pytest.mark.parametrize("tile", ["128x128", "128x256", "128x512"])
def test_conv_u8_gather_tiles(sq, oracle, tuning, tile):
    """Gather-kernel tiles with the byte output (the widest tile has none: the library picks the next one)."""
    tuning(f"path=gather,tile={tile}")
    check_layer_u8(sq, oracle, S.ConvLayer("u8_tiles", 1, 9, 31, 96, 520, 3, 3, (1, 1), (1, 1)), S.Mode(4, S.OPT3, 1, 1), seed_cfg=9)


def test_conv_u8_chain(sq, oracle):
    """Two layers chained on the device: the first layer's bytes are the second layer's NHWC input."""
    l1 = S.ConvLayer("chain1", 2, 12, 12, 64, 96, 3, 3, (1, 1), (1, 1))
    l2 = S.ConvLayer("chain2", 2, 12, 12, 96, 40, 1, 1, index=1)
    mode = S.Mode(4, S.OPT5, 1, 1)
    x, w1, _ = S.gen_layer(9, l1)
    _, w2, _ = S.gen_layer(9, l2)
    f1, f2 = S.gen_requant(l1, S.rng_for(9, 950)), S.gen_requant(l2, S.rng_for(9, 951))
    y1 = run_conv_u8(sq, x, w1, f1, l1, mode)
    y2 = run_conv_u8(sq, y1.reshape(l2.x_shape()), w2, f2, l2, mode)
    r1 = oracle.conv_gemm_u8(x, w1, f1, l1.stride, l1.pad, **mode.kwargs())
    r2 = oracle.conv_gemm_u8(r1.reshape(l2.x_shape()), w2, f2, l2.stride, l2.pad, **mode.kwargs())
    assert np.array_equal(y1, r1) and np.array_equal(y2, r2)


@pytest.mark.parametrize("tn", ["64", "128", "256"])
def test_conv_patch_channel_tiles(sq, oracle, tuning, tn):
    """Every output-channel tile width of the input-patch kernel on the same layer."""
    tuning(f"path=patch,patch_tn={tn}")
    check_layer(sq, oracle, S.ConvLayer("p_tn", 3, 14, 14, 128, 520, 3, 3, (1, 1), (1, 1)), S.Mode(4, S.OPT5, 1, 1), seed_cfg=9)


WIDE_TILE_LAYERS = [
    # reduction steps (64 indices each) per tile: 1, 2, 3, 4, 5 -- every remainder of the four-step unrolled loop
    S.ConvLayer("wide_1x1_c64", 1, 9, 31, 64, 300),
    S.ConvLayer("wide_1x1_c128", 1, 9, 31, 128, 300),
    S.ConvLayer("wide_1x1_c192", 2, 8, 9, 192, 512),
    S.ConvLayer("wide_1x1_c256", 1, 5, 27, 256, 260),
    S.ConvLayer("wide_1x1_c320", 1, 5, 27, 320, 900),          # two output-channel tiles, the second ragged
    # several taps with zero padding at the borders; 96 channels leave a tap's last chunks in its channel padding
    S.ConvLayer("wide_3x3_c64", 2, 12, 12, 64, 384, 3, 3, (1, 1), (1, 1)),
    S.ConvLayer("wide_3x3s2_c96", 1, 13, 17, 96, 300, 3, 3, (2, 2), (1, 1)),
    S.ConvLayer("wide_5x1_c80", 1, 11, 9, 80, 257, 5, 1, (1, 1), (2, 0)),
    S.ConvLayer("wide_1x1s2_c512", 1, 15, 15, 512, 300, 1, 1, (2, 2), (0, 0)),
]


@pytest.mark.parametrize("mode", [S.Mode(4, S.OPT5, 1, 1), S.Mode(4, S.OPT3, 0, 1), S.Mode(3, S.OPT6_3B, 1, 1), S.Mode(2, S.OPT7_2B, 0, 0), S.PLAIN8],
                         ids=lambda m: m.label + f"-{m.shift_mask:#x}")
@pytest.mark.parametrize("layer", WIDE_TILE_LAYERS, ids=lambda l: l.name)
def test_conv_widest_gather_tile(sq, oracle, tuning, layer, mode):
    """The 128 x 512 tile of the gather kernel (main loop pipelined by half steps, taps tracked in scalar
    registers) on every loop remainder, on multi-tap layers with padding, and on channel-padded taps."""
    tuning("path=gather,tile=128x512")
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    assert "tile=128x512" in sq.sparq_conv_plan(d, sq.mode(*mode.astuple()))
    check_layer(sq, oracle, layer, mode, seed_cfg=9)


def test_widest_gather_tile_needs_step_aligned_taps(sq, tuning):
    """With at most 32 channels a tap is shorter than a reduction step: the library takes the next tile."""
    tuning("path=gather,tile=128x512")
    d = sq.conv_desc(1, 9, 9, 32, 300, 3, 3, (1, 1), (1, 1))
    assert "tile=128x256" in sq.sparq_conv_plan(d, sq.mode(4, S.OPT5, 1, 1))


@pytest.mark.parametrize("mode", MODES_N4 + MODES_LOW + MODES_ODD, ids=lambda m: m.label + f"-{m.shift_mask:#x}")
def test_conv_all_modes(sq, oracle, mode, path):
    check_layer(sq, oracle, S.ConvLayer("3x3_modes", 1, 14, 14, 64, 48, 3, 3, (1, 1), (1, 1), index=3), mode)


def test_extreme_values(sq, oracle):
    """Saturation and accumulator extremes: all-255 / all-zero activations, all -127 / +127 weights, K = 4608."""
    layer = S.ConvLayer("extreme", 1, 70, 1, 4608, 8)
    sc = np.full(8, 0.005, dtype=np.float32)
    for xv in (255, 0, 128):
        for wv in (-127, 127):
            x = np.full(layer.x_shape(), xv, dtype=np.uint8)
            w = np.full(layer.w_shape(), wv, dtype=np.int8)
            for mode in (S.Mode(4, S.OPT5, 1, 1), S.PLAIN8):
                acc, _ = run_conv(sq, x, w, sc, layer, mode)
                ref, _ = oracle.conv_gemm(x, w, **mode.kwargs())
                assert np.array_equal(acc, ref)


def test_only_out_or_only_acc(sq, oracle):
    layer = S.ConvLayer("3x3_outs", 1, 9, 9, 32, 16, 3, 3, (1, 1), (1, 1))
    mode = S.Mode(4, S.OPT5, 1, 1)
    x, w, sc = S.gen_layer(8, layer)
    ref_acc, ref_out = oracle.conv_gemm(x, w, layer.stride, layer.pad, scale=sc, **mode.kwargs())
    acc, _ = run_conv(sq, x, w, sc, layer, mode, want_acc=True, want_out=False)
    assert np.array_equal(acc, ref_acc)
    _, out = run_conv(sq, x, w, sc, layer, mode, want_acc=False, want_out=True)
    assert np.all(np.abs(out.astype(np.float64) - ref_out) <= 1e-6 * np.abs(ref_out))


def test_fused_equals_trim_then_plain(sq):
    """GPU-internal cross-check: trimming with the standalone kernel and contracting at plain
    8 bits gives the same accumulators as the fused kernel."""
    layer = S.ConvLayer("3x3_x", 2, 12, 12, 64, 40, 3, 3, (1, 1), (1, 1))
    mode = S.Mode(4, S.OPT3, 1, 1)
    x, w, sc = S.gen_layer(8, layer)
    fused, _ = run_conv(sq, x, w, sc, layer, mode, want_out=False)
    xd = dev(x)
    y = torch.empty_like(xd)
    sq.sparq_trim(xd, y, sq.mode(*mode.astuple()))
    torch.cuda.synchronize()
    plain, _ = run_conv(sq, y.cpu().numpy(), w, sc, layer, S.PLAIN8, want_out=False)
    assert np.array_equal(fused, plain)
