"""Pins for the oracle's trimmed convolution and dequantisation (CPU only)."""
import numpy as np
import pytest
import torch

import sparq_second_opinion as so
import sparq_synth as S


def _table_trim(x, n, mask, rnd, pairing):
    """Trim an NHWC tensor with the separately written formulation (slow, tiny inputs only)."""
    y = np.empty_like(x)
    flat_x = x.reshape(-1, x.shape[-1])
    flat_y = y.reshape(-1, x.shape[-1])
    C = x.shape[-1]
    for r in range(flat_x.shape[0]):
        for c in range(0, C, 2):
            a = int(flat_x[r, c])
            b = int(flat_x[r, c + 1]) if c + 1 < C else 0
            ta, tb = so.pair(a, b, n, mask, rnd, pairing)
            flat_y[r, c] = ta
            if c + 1 < C:
                flat_y[r, c + 1] = tb
    return y


def _torch_conv(x_u8, w_i8, stride, pad):
    """Library convolution in float64 (exact for these magnitudes), NHWC in / [M,N] out."""
    xt = torch.from_numpy(x_u8.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w_i8.astype(np.float64)).permute(0, 3, 1, 2)
    y = torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad)
    return y.permute(0, 2, 3, 1).reshape(-1, w_i8.shape[0]).numpy().round().astype(np.int64)


CASES = [
    # B, H, W, C, N, KH, KW, stride, pad
    (1, 5, 5, 4, 3, 3, 3, (1, 1), (1, 1)),
    (2, 7, 6, 5, 4, 3, 3, (2, 2), (1, 1)),
    (1, 9, 8, 6, 5, 1, 7, (1, 1), (0, 3)),
    (1, 8, 9, 3, 2, 7, 1, (1, 1), (3, 0)),
    (2, 6, 6, 8, 7, 1, 1, (2, 2), (0, 0)),
    (1, 11, 11, 2, 3, 5, 5, (1, 1), (2, 2)),
    (1, 12, 10, 3, 4, 7, 7, (2, 2), (3, 3)),
    (3, 4, 4, 16, 9, 3, 3, (1, 1), (0, 0)),
]


@pytest.mark.parametrize("case", CASES)
def test_plain_8bit_equals_library_convolution(oracle, case):
    """window_bits = 8 reduces to an ordinary integer convolution."""
    B, H, W, C, N, KH, KW, st, pd = case
    rng = S.rng_for(7, 1)
    x = S.gen_activations((B, H, W, C), 0.4, rng)
    w = S.gen_weights((N, KH, KW, C), rng)
    acc, _ = oracle.conv_gemm(x, w, st, pd, window_bits=8, shift_mask=1, round_nearest=0, pair=0)
    assert np.array_equal(acc.astype(np.int64), _torch_conv(x, w, st, pd))


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("mode", [(4, 0x1F, 1, 1), (4, 0x15, 0, 1), (4, 0x11, 1, 0), (2, 0x7F, 1, 1), (3, 0x3F, 0, 1)])
def test_trimmed_conv_equals_library_conv_of_trimmed_tensor(oracle, case, mode):
    """The trim applies to input elements, so it commutes with the im2col gather:
    oracle(x) == library_conv(separately trimmed x)."""
    B, H, W, C, N, KH, KW, st, pd = case
    n, mask, rnd, pairing = mode
    rng = S.rng_for(7, 2)
    x = S.gen_activations((B, H, W, C), 0.5, rng)
    w = S.gen_weights((N, KH, KW, C), rng)
    acc, _ = oracle.conv_gemm(x, w, st, pd, window_bits=n, shift_mask=mask, round_nearest=rnd, pair=pairing)
    xt = _table_trim(x, n, mask, rnd, pairing)
    assert np.array_equal(acc.astype(np.int64), _torch_conv(xt, w, st, pd))


def test_tiny_conv_by_hand_loops(oracle):
    """1x5x5x4 -> 3 channels, 3x3 pad 1, nested Python loops with the pair rule inline."""
    rng = S.rng_for(7, 3)
    x = S.gen_activations((1, 5, 5, 4), 0.5, rng)
    w = S.gen_weights((3, 3, 3, 4), rng)
    acc, _ = oracle.conv_gemm(x, w, (1, 1), (1, 1), window_bits=4, shift_mask=0x1F, round_nearest=1, pair=1)
    exp = np.zeros((25, 3), dtype=np.int64)
    for oy in range(5):
        for ox in range(5):
            for n in range(3):
                tot = 0
                for kh in range(3):
                    for kw in range(3):
                        iy, ix = oy - 1 + kh, ox - 1 + kw
                        if not (0 <= iy < 5 and 0 <= ix < 5):
                            continue
                        for c in range(0, 4, 2):
                            a, b = int(x[0, iy, ix, c]), int(x[0, iy, ix, c + 1])
                            ta, tb = so.pair(a, b, 4, 0x1F, 1, 1)
                            tot += ta * int(w[n, kh, kw, c]) + tb * int(w[n, kh, kw, c + 1])
                exp[oy * 5 + ox, n] = tot
    assert np.array_equal(acc, exp)


def test_row_selection_matches_full(oracle):
    rng = S.rng_for(7, 4)
    x = S.gen_activations((2, 9, 9, 6), 0.5, rng)
    w = S.gen_weights((5, 3, 3, 6), rng)
    full, _ = oracle.conv_gemm(x, w, (2, 2), (1, 1))
    rows = np.array([0, 3, 24, 25, 49, 7], dtype=np.int64)
    part, _ = oracle.conv_gemm(x, w, (2, 2), (1, 1), rows=rows)
    assert full.shape == (2 * 5 * 5, 5)
    assert np.array_equal(part, full[rows])


def test_sparq_error_bound_against_exact_product(oracle):
    """|trimmed dot product - exact| <= sum |w| * (2^s - 1): the paper's claim that only the
    dropped LSBs are lost; with pairing on, values next to a zero contribute no error at all."""
    rng = S.rng_for(7, 5)
    x = S.gen_activations((1, 64, 1, 128), 0.5, rng)
    w = S.gen_weights((8, 1, 1, 128), rng)
    exact, _ = oracle.conv_gemm(x, w, window_bits=8, shift_mask=1, round_nearest=0, pair=0)
    xv = x.reshape(64, 128).astype(np.int64)
    wv = w.reshape(8, 128).astype(np.int64)
    assert np.array_equal(exact, xv @ wv.T)
    lsb = np.maximum(0, np.floor(np.log2(np.maximum(xv, 1))).astype(np.int64) - 3)   # 5opt shift
    for pairing in (0, 1):
        got, _ = oracle.conv_gemm(x, w, window_bits=4, shift_mask=0x1F, round_nearest=0, pair=pairing)
        slack = (2 ** lsb - 1)
        if pairing:
            partner = xv.reshape(64, 64, 2)[:, :, ::-1].reshape(64, 128)
            slack = np.where(partner == 0, 0, slack)
        bound = slack @ np.abs(wv).T
        assert np.all(np.abs(got.astype(np.int64) - exact) <= bound)
    # all pairs contain a zero -> exact
    xz = x.copy()
    xz[..., 1::2] = 0
    a, _ = oracle.conv_gemm(xz, w, window_bits=4, shift_mask=0x11, round_nearest=0, pair=1)
    b, _ = oracle.conv_gemm(xz, w, window_bits=8, shift_mask=1, round_nearest=0, pair=0)
    assert np.array_equal(a, b)


def test_accumulator_extremes(oracle):
    """All-255 activations with all -127 weights at K = 4608: sums stay inside int32 and are exact."""
    x = np.full((1, 2, 1, 4608), 255, dtype=np.uint8)
    w = np.full((2, 1, 1, 4608), -127, dtype=np.int8)
    acc, _ = oracle.conv_gemm(x, w, window_bits=4, shift_mask=0x1F, round_nearest=1, pair=1)
    assert np.all(acc == 240 * -127 * 4608)
    acc, _ = oracle.conv_gemm(x, w, window_bits=8, shift_mask=1, round_nearest=0, pair=0)
    assert np.all(acc == 255 * -127 * 4608)


def test_dequant(oracle):
    rng = S.rng_for(7, 6)
    acc = rng.integers(-2 ** 31, 2 ** 31, size=(37, 19), dtype=np.int64).astype(np.int32)
    acc[0, 0], acc[0, 1], acc[0, 2] = 2 ** 31 - 1, -2 ** 31, 0
    sc = S.gen_scales(19, rng)
    out = oracle.dequant(acc, sc)
    assert out.dtype == np.float64
    assert np.array_equal(out, acc.astype(np.float64) * sc.astype(np.float64)[None, :])
    # and the fused output of the conv entry point is the same operation
    x = S.gen_activations((1, 6, 6, 4), 0.5, rng)
    w = S.gen_weights((19, 3, 3, 4), rng)
    a, o = oracle.conv_gemm(x, w, (1, 1), (1, 1), scale=sc)
    assert np.array_equal(o, oracle.dequant(a, sc))


def test_config0_shape_and_sanity(oracle):
    """Config 0 end to end on the CPU: M=3136, K=576, N=64; cross-checked on sampled rows with numpy."""
    (layer,) = S.config0()
    assert (layer.M, layer.K, layer.N) == (3136, 576, 64)
    x, w, sc = S.gen_layer(0, layer)
    acc, out = oracle.conv_gemm(x, w, layer.stride, layer.pad, scale=sc, **layer.mode.kwargs())
    assert acc.shape == (3136, 64)
    xt = oracle.trim(x, **layer.mode.kwargs())
    xp = np.pad(xt.astype(np.int64), ((0, 0), (1, 1), (1, 1), (0, 0)))
    for m in (0, 55, 56, 1567, 3080, 3135):
        oy, ox = divmod(m, 56)
        patch = xp[0, oy:oy + 3, ox:ox + 3, :].reshape(-1)
        assert np.array_equal(acc[m], w.reshape(64, -1).astype(np.int64) @ patch)
    assert np.allclose(out, acc * sc.astype(np.float64)[None, :], rtol=0, atol=0)
