"""Pins of the oracle's 2:4 weight-sparse convolution (CPU only): activations picked by the kept weights' coordinates,
the picked two forming the vSPARQ pair (Section 4, sparse tensor core; Section 5.3)."""
import numpy as np
import pytest

import sparq_synth as S

FLOOR5 = dict(window_bits=4, shift_mask=S.OPT5, round_nearest=0, pair=1)


def one_group(oracle, x4, idx, vals, **mode):
    """acc of a 1x1 'convolution' over one pixel with four channels and one output channel."""
    x = np.array(x4, np.uint8).reshape(1, 1, 1, 4)
    acc, _ = oracle.conv_gemm_sparse24(x, np.array(vals, np.int8).reshape(1, 1, 1, 2), np.array(idx, np.uint8).reshape(1, 1, 1, 2), **mode)
    return int(acc[0, 0])


def test_hand_worked_groups(oracle):
    """Group (27, 0, 5, 200), 5opt, plain trim.  27 alone trims to 26 (the paper's example, Section 3.1), 200 = 11001000b
    to 192, 5 stays; next to a zero a value keeps all eight bits (Eq. 2)."""
    g = (27, 0, 5, 200)
    assert one_group(oracle, g, (0, 1), (3, 7), **FLOOR5) == 27 * 3 + 0 * 7            # partner 0 -> 27 untouched
    assert one_group(oracle, g, (0, 2), (3, 7), **FLOOR5) == 26 * 3 + 5 * 7            # both non-zero -> both trimmed
    assert one_group(oracle, g, (0, 3), (3, -7), **FLOOR5) == 26 * 3 - 192 * 7
    assert one_group(oracle, g, (1, 3), (3, 7), **FLOOR5) == 0 * 3 + 200 * 7           # 200 keeps its eight bits
    assert one_group(oracle, g, (2, 3), (1, 1), **FLOOR5) == 5 + 192
    # the same activation, another output channel's coordinates: 200 is trimmed in one and not in the other
    assert one_group(oracle, g, (1, 3), (0, 1), **FLOOR5) - one_group(oracle, g, (2, 3), (0, 1), **FLOOR5) == 8
    # a kept weight that is zero still names the partner: (27 | 5) trims 27, (27 | 0) does not
    assert one_group(oracle, g, (0, 2), (1, 0), **FLOOR5) == 26 and one_group(oracle, g, (0, 1), (1, 0), **FLOOR5) == 27
    # vSPARQ off: every picked value is trimmed on its own
    assert one_group(oracle, g, (0, 1), (1, 1), window_bits=4, shift_mask=S.OPT5, round_nearest=0, pair=0) == 26
    # rounding: 27 -> 28
    assert one_group(oracle, g, (0, 2), (1, 0), window_bits=4, shift_mask=S.OPT5, round_nearest=1, pair=1) == 28


def test_bad_coordinates_are_rejected(oracle):
    x = np.zeros((1, 1, 1, 4), np.uint8)
    v = np.ones((1, 1, 1, 2), np.int8)
    for idx in ((1, 1), (2, 1), (0, 4)):
        with pytest.raises(ValueError):
            oracle.conv_gemm_sparse24(x, v, np.array(idx, np.uint8).reshape(1, 1, 1, 2), **FLOOR5)
    with pytest.raises(ValueError):                                   # C not a multiple of 4
        oracle.conv_gemm_sparse24(np.zeros((1, 1, 1, 6), np.uint8), np.ones((1, 1, 1, 3), np.int8), np.zeros((1, 1, 1, 3), np.uint8), **FLOOR5)


@pytest.mark.parametrize("mode", [S.Mode(4, S.OPT5, 1, 0), S.Mode(4, S.OPT3, 0, 0), S.Mode(8, 1, 0, 0), S.Mode(2, S.OPT7_2B, 1, 0)], ids=lambda m: m.label)
def test_without_pairing_it_is_the_dense_convolution_on_the_decompressed_weights(oracle, mode):
    """vSPARQ off (or a plain 8-bit layer): the coordinates only say where the zeros are."""
    rng = S.rng_for(9, 1)
    x = S.gen_activations((2, 9, 8, 16), 0.5, rng)
    wv, wi = S.gen_sparse24_weights((5, 3, 3, 16), rng)
    got, _ = oracle.conv_gemm_sparse24(x, wv, wi, (1, 1), (1, 1), **mode.kwargs())
    want, _ = oracle.conv_gemm(x, S.sparse24_to_dense(wv, wi), (1, 1), (1, 1), **mode.kwargs())
    assert np.array_equal(got, want)


@pytest.mark.parametrize("mode", [S.Mode(4, S.OPT5, 1, 1), S.Mode(4, S.OPT2, 0, 1), S.Mode(3, S.OPT6_3B, 1, 1)], ids=lambda m: m.label)
def test_natural_pairs_reduce_to_the_dense_trimmed_convolution(oracle, mode):
    """When every group keeps positions (0,1) or (2,3) the picked pair is a pair of consecutive channels (2j, 2j+1):
    the result is the ordinary SPARQ convolution with the decompressed weights (the other pair meets zero weights)."""
    rng = S.rng_for(9, 2)
    x = S.gen_activations((2, 7, 9, 24), 0.5, rng)
    wv, wi = S.gen_sparse24_weights((6, 3, 1, 24), rng, natural_pairs=True)
    sc = S.gen_scales(6, rng)
    got, gout = oracle.conv_gemm_sparse24(x, wv, wi, (2, 1), (1, 0), scale=sc, **mode.kwargs())
    want, wout = oracle.conv_gemm(x, S.sparse24_to_dense(wv, wi), (2, 1), (1, 0), scale=sc, **mode.kwargs())
    assert np.array_equal(got, want) and np.array_equal(gout, wout)


def test_against_nested_loops(oracle):
    """A small strided, padded convolution by Python loops; the pair rule itself comes from the (pinned) standalone trim."""
    rng = S.rng_for(9, 3)
    mode = S.Mode(4, S.OPT3, 1, 1)
    B, H, W, C, N, KH, KW, sh, sw, ph, pw = 2, 6, 5, 8, 3, 3, 2, 2, 1, 1, 1
    x = S.gen_activations((B, H, W, C), 0.4, rng)
    wv, wi = S.gen_sparse24_weights((N, KH, KW, C), rng)
    Ho, Wo = (H + 2 * ph - KH) // sh + 1, (W + 2 * pw - KW) // sw + 1
    want = np.zeros((B * Ho * Wo, N), np.int64)
    for b in range(B):
        for oy in range(Ho):
            for ox in range(Wo):
                for n in range(N):
                    s = 0
                    for kh in range(KH):
                        for kw_ in range(KW):
                            iy, ix = oy * sh - ph + kh, ox * sw - pw + kw_
                            if not (0 <= iy < H and 0 <= ix < W):
                                continue
                            for g in range(C // 4):
                                i0, i1 = wi[n, kh, kw_, 2 * g], wi[n, kh, kw_, 2 * g + 1]
                                pair = np.array([[x[b, iy, ix, 4 * g + i0], x[b, iy, ix, 4 * g + i1]]], np.uint8)
                                t = oracle.trim(pair, **mode.kwargs())[0].astype(int)
                                s += t[0] * int(wv[n, kh, kw_, 2 * g]) + t[1] * int(wv[n, kh, kw_, 2 * g + 1])
                    want[(b * Ho + oy) * Wo + ox, n] = s
    got, _ = oracle.conv_gemm_sparse24(x, wv, wi, (sh, sw), (ph, pw), **mode.kwargs())
    assert np.array_equal(got, want)
    rows = np.array([0, 5, len(want) - 1])
    sub, _ = oracle.conv_gemm_sparse24(x, wv, wi, (sh, sw), (ph, pw), rows=rows, **mode.kwargs())
    assert np.array_equal(sub, want[rows])


def test_error_bound_against_the_untrimmed_sparse_convolution(oracle):
    """Every picked activation is off by less than its window's LSB (at most 15 for 4-bit windows)."""
    rng = S.rng_for(9, 4)
    x = S.gen_activations((1, 5, 5, 32), 0.3, rng)
    wv, wi = S.gen_sparse24_weights((4, 1, 1, 32), rng)
    exact, _ = oracle.conv_gemm_sparse24(x, wv, wi, window_bits=8, shift_mask=1, round_nearest=0, pair=0)
    got, _ = oracle.conv_gemm_sparse24(x, wv, wi, **FLOOR5)
    bound = 15 * np.abs(wv.astype(np.int64)).reshape(4, -1).sum(1)
    assert np.all(np.abs(got.astype(np.int64) - exact) <= bound[None, :]) and not np.array_equal(got, exact)
