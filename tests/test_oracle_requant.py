"""Pins of the oracle's requantisation (Section 5, first paragraph: unsigned per-layer activation quantisation).

The operation is defined by its arithmetic -- int32 -> fp32, one fp32 product, round to nearest integer with ties
to even, clamp to [0, 255] -- so the pins are independent statements of that arithmetic: hand-worked ties and
clamps, exact rational arithmetic with IEEE-754 rounding written out on fractions, and structural properties.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def rne_int(q: Fraction) -> int:
    """Nearest integer, ties to even, on an exact rational."""
    f = q.numerator // q.denominator          # floor
    r = q - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return f


def to_fp32(q: Fraction) -> Fraction:
    """Nearest binary32 value (24-bit significand, ties to even) of an exact rational in the normal range."""
    if q == 0:
        return q
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = 0
    while a >= 1 << 24:
        a /= 2
        e += 1
    while a < 1 << 23:
        a *= 2
        e -= 1
    assert -149 < e < 104                       # no subnormals, no overflow in these tests
    return sign * Fraction(rne_int(a)) * (Fraction(2) ** e)


def requant_exact(acc: int, factor: float) -> int:
    p = to_fp32(to_fp32(Fraction(acc)) * Fraction(factor))     # Fraction(float) is exact
    return min(max(rne_int(p), 0), 255)


def test_hand_worked_ties_and_clamps():
    acc = np.array([[3, 5, 1, -7, 7, 1000, 255, 256, 0, -1, 509, 511]], dtype=np.int32)
    got = oracle.requant(acc, np.full(12, 0.5, dtype=np.float32))
    #            1.5 2.5 0.5 -3.5 3.5 500  127.5 128 0  -0.5 254.5 255.5
    assert got.tolist() == [[2, 2, 0, 0, 4, 255, 128, 128, 0, 0, 254, 255]]


def test_unit_factor_is_a_clamp():
    acc = np.arange(-300, 600, dtype=np.int32).reshape(-1, 4)
    got = oracle.requant(acc, np.ones(4, dtype=np.float32))
    assert np.array_equal(got, np.clip(acc, 0, 255).astype(np.uint8))


def test_factor_is_per_output_channel():
    acc = np.full((3, 4), 100, dtype=np.int32)
    got = oracle.requant(acc, np.array([1.0, 0.5, 0.25, 2.0], dtype=np.float32))
    assert got.tolist() == [[100, 50, 25, 200]] * 3


def test_exact_products_against_rational_arithmetic():
    """Factors k/256 with 12-bit k and 12-bit |acc|: the product is exact in fp32, only the tie rule matters."""
    rng = np.random.default_rng(5)
    acc = rng.integers(-4095, 4096, size=(64, 32), dtype=np.int32)
    k = rng.integers(1, 4096, size=32)
    factor = (k / 256.0).astype(np.float32)
    got = oracle.requant(acc, factor)
    for m in range(acc.shape[0]):
        for n in range(32):
            q = Fraction(int(acc[m, n]) * int(k[n]), 256)
            assert got[m, n] == min(max(rne_int(q), 0), 255)


def test_general_values_against_ieee_rounding_on_fractions():
    """Accumulators beyond 2^24 (inexact int -> fp32) and arbitrary fp32 factors (inexact products)."""
    rng = np.random.default_rng(6)
    acc = np.concatenate([rng.integers(-(1 << 31), (1 << 31) - 1, size=200), rng.integers(-70000, 70000, size=400),
                          np.array([0, 1, -1, (1 << 24) + 1, (1 << 24) + 3, (1 << 31) - 1, -(1 << 31), 16777217, 33554434 + 2])])
    acc = acc.astype(np.int32).reshape(-1, 1)
    for f in (3.1e-3, 1.9073486e-6, 7.6e-8, 0.0123456, 1.0 / 3.0, 0.0039215689):
        factor = np.array([f], dtype=np.float32)
        got = oracle.requant(acc, factor)
        for a, g in zip(acc[:, 0].tolist(), got[:, 0].tolist()):
            assert g == requant_exact(a, float(factor[0])), (a, f)


def test_half_way_products_that_need_the_fp32_rounding_first():
    """(2^24 + 1) * 2^-17 = 128.0000076...: the int -> fp32 step rounds 2^24 + 1 to 2^24 first."""
    acc = np.array([[(1 << 24) + 1, (1 << 24) + 3]], dtype=np.int32)
    got = oracle.requant(acc, np.full(2, 2.0 ** -17, dtype=np.float32))
    assert got.tolist() == [[128, 128]]
    # (2^24 + 1) * 2.5 * 2^-24: exactly 2.5 after the int -> fp32 step (tie, to even: 2), 2.50000015 without it (3)
    got = oracle.requant(np.array([[(1 << 24) + 1, 1 << 24, (1 << 24) + 2]], dtype=np.int32),
                         np.full(3, 2.5 * 2.0 ** -24, dtype=np.float32))
    assert got.tolist() == [[2, 2, 3]]
    # 2^-23 is a power of two, so these products are exact: 1.50000012 -> 2, 1.5 (tie) -> 2, 0.5 (tie) -> 0, 0.50000012 -> 1
    got = oracle.requant(np.array([[12582913, 12582912, 4194304, 4194305]], dtype=np.int32), np.full(4, 2.0 ** -23, dtype=np.float32))
    assert got.tolist() == [[2, 2, 0, 1]]
    # 2^25 + 2 -> fp32 keeps it (even significand), 2^25 + 6 rounds to 2^25 + 8
    acc = np.array([[(1 << 25) + 2, (1 << 25) + 6]], dtype=np.int32)
    got = oracle.requant(acc, np.full(2, 2.0 ** -20, dtype=np.float32))
    assert got.tolist() == [[32, 32]]


@pytest.mark.parametrize("f", [0.003, 0.02, 0.7])
def test_monotone_and_zero_below_zero(f):
    acc = np.arange(-2000, 40000, 7, dtype=np.int32).reshape(-1, 1)
    got = oracle.requant(acc, np.array([f], dtype=np.float32))[:, 0].astype(int)
    assert np.all(np.diff(got) >= 0)
    assert np.all(got[acc[:, 0] <= 0] == 0)
    assert got[-1] == min(255, rne_int(to_fp32(Fraction(int(acc[-1, 0])) * Fraction(float(np.float32(f))))))


def test_conv_gemm_u8_is_requant_of_the_accumulators():
    rng = np.random.default_rng(7)
    x = rng.integers(0, 256, size=(2, 6, 5, 8), dtype=np.uint8)
    w = rng.integers(-127, 128, size=(5, 3, 3, 8), dtype=np.int8)
    factor = rng.uniform(1e-3, 6e-3, size=5).astype(np.float32)
    kw = dict(window_bits=4, shift_mask=0x1F, round_nearest=1, pair=1)
    acc, _ = oracle.conv_gemm(x, w, (1, 1), (1, 1), **kw)
    y = oracle.conv_gemm_u8(x, w, factor, (1, 1), (1, 1), **kw)
    assert y.dtype == np.uint8 and y.shape == acc.shape
    assert np.array_equal(y, oracle.requant(acc, factor))
    assert 0 < np.count_nonzero(y) < y.size and y.max() > 100          # the case exercises both clamps' neighbourhood


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        oracle.requant(np.zeros((2, 0), dtype=np.int32), np.zeros(0, dtype=np.float32))
