"""Pins for the oracle's bSPARQ / vSPARQ trim (CPU only).

Each test checks the oracle against something other than itself: values the
paper prints, closed forms derived by hand from the definition, invariants the
method must satisfy, an independently written value-range formulation, or
brute force over the whole input domain.
"""
import os

import numpy as np
import pytest

import sparq_second_opinion as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_examples.txt")

N4_MASKS = {"5opt": 0x1F, "3opt": 0x15, "2opt": 0x11}
ALL_N4_MASKS = [0x11 | (sub << 1) for sub in range(8)]
LOW_BIT = {"3b-6opt": (3, 0x3F), "2b-7opt": (2, 0x7F)}


def all_modes():
    for mask in ALL_N4_MASKS:
        yield 4, mask
    for n, mask in LOW_BIT.values():
        yield n, mask
    yield 3, 0x21 | 0x08     # 3-bit windows at shifts {0,3,5}
    yield 2, 0x55            # 2-bit windows at shifts {0,2,4,6}


def test_paper_worked_examples(oracle):
    """Section 3.1 prints these window positions / values."""
    rows = 0
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            x, n, mask, rnd, val, shift = (int(t, 0) for t in line.split())
            assert oracle.trim_value(x, n, mask, rnd) == (val, shift)
            rows += 1
    assert rows == 5


@pytest.mark.parametrize("n,mask", list(all_modes()))
@pytest.mark.parametrize("rnd", [0, 1])
def test_matches_value_range_formulation(oracle, n, mask, rnd):
    """All 256 values against the grid/region description written separately."""
    for x in range(256):
        got, s = oracle.trim_value(x, n, mask, rnd)
        assert got == so.trim(x, n, mask, rnd), (x, n, hex(mask), rnd)
        if x:
            assert 2 ** s == so.region_step(x, n, mask)


@pytest.mark.parametrize("n,mask", list(all_modes()))
@pytest.mark.parametrize("rnd", [0, 1])
def test_invariants(oracle, n, mask, rnd):
    prev = -1
    for x in range(256):
        t, s = oracle.trim_value(x, n, mask, rnd)
        assert 0 <= t <= 255
        if x == 0:
            assert t == 0                                   # zero stays zero
        if x < 2 ** n:
            assert t == x                                   # fits the window at shift 0
        # at most n significant bits: msb - lsb + 1 <= n
        if t:
            msb = t.bit_length() - 1
            lsb = (t & -t).bit_length() - 1
            assert msb - lsb + 1 <= n
            assert lsb >= s and msb <= s + n - 1            # ... and inside the chosen window
        assert (mask >> s) & 1                              # an allowed placement
        assert abs(x - t) < 2 ** s or s == 0 and t == x     # error below the window's LSB
        if rnd == 0:
            assert t <= x
        assert t >= prev                                    # monotone
        prev = t
        assert oracle.trim_value(t, n, mask, rnd)[0] == t   # idempotent


def test_values_below_16_unchanged_and_5opt_regions(oracle):
    """x < 16 is exact for every 4-bit option set; 5opt regions are
    [0,15],[16,31],[32,63],[64,127],[128,255] with shifts 0..4."""
    for mask in ALL_N4_MASKS:
        for rnd in (0, 1):
            for x in range(16):
                assert oracle.trim_value(x, 4, mask, rnd) == (x, 0)
    for x in range(1, 256):
        expect = max(0, x.bit_length() - 4)
        assert oracle.trim_value(x, 4, 0x1F, 0)[1] == expect


def test_region_counts(oracle):
    """Section 3.1: up to five regions for 4-bit activations, six for 3-bit, seven for 2-bit."""
    def regions(n, mask):
        return len({oracle.trim_value(x, n, mask, 0)[1] for x in range(1, 256)})
    assert regions(4, 0x1F) == 5
    assert regions(4, 0x15) == 3
    assert regions(4, 0x11) == 2
    assert regions(3, 0x3F) == 6
    assert regions(2, 0x7F) == 7


def test_2opt_is_msb_or_lsb_nibble(oracle):
    """2opt keeps either bits [7:4] or bits [3:0] (Section 3.1), i.e. the halves of Eq. 3."""
    for x in range(256):
        t, _ = oracle.trim_value(x, 4, 0x11, 0)
        assert t == (x if x < 16 else (x // 16) * 16)
        hi, lo = x // 16, x % 16
        assert 16 * hi + lo == x                            # Eq. 3 with w = 1
        assert t in (16 * hi, lo)


def _closed_form_floor_error(n, shifts):
    """Sum over x of x - T(x), plain trim: in the region with step 2**t the
    residual x mod 2**t is uniform, each residual value occurring
    (region size) / 2**t times."""
    total, lo = 0, 0
    for t in shifts:
        hi = 2 ** (t + n)
        size = hi - lo
        total += (size // 2 ** t) * sum(range(2 ** t))
        lo = hi
    return total


def _closed_form_round_error(n, shifts):
    """Sum over x of |x - T(x)| with rounding: residual r costs min(r, 2**t - r),
    except in the top code q = 2**n - 1 where rounding up is impossible and the
    cost is r itself: an extra h*(h-1), h = 2**(t-1), per region."""
    total, lo = 0, 0
    for t in shifts:
        hi = 2 ** (t + n)
        size = hi - lo
        step = 2 ** t
        total += (size // step) * sum(min(r, step - r) for r in range(step))
        if t > 0:
            h = step // 2
            total += h * (h - 1)
        lo = hi
    return total


@pytest.mark.parametrize("name,shifts", [("5opt", [0, 1, 2, 3, 4]), ("3opt", [0, 2, 4]), ("2opt", [0, 4])])
def test_closed_form_error_sums(oracle, name, shifts):
    mask = N4_MASKS[name]
    fl = sum(x - oracle.trim_value(x, 4, mask, 0)[0] for x in range(256))
    rd = sum(abs(x - oracle.trim_value(x, 4, mask, 1)[0]) for x in range(256))
    assert fl == _closed_form_floor_error(4, shifts)
    assert rd == _closed_form_round_error(4, shifts)
    # hand-evaluated numbers: 8*(1+6+28+120), 72+1440, 15*120
    assert fl == {"5opt": 1240, "3opt": 1512, "2opt": 1800}[name]
    assert rd == {"5opt": 750, "3opt": 874, "2opt": 1016}[name]
    # image sizes: 16 exact values + (2**n - 2**n / 2**(gap)) codes per further region
    image = {oracle.trim_value(x, 4, mask, 0)[0] for x in range(256)}
    assert len(image) == {"5opt": 48, "3opt": 40, "2opt": 31}[name]
    assert image == {oracle.trim_value(x, 4, mask, 1)[0] for x in range(256)}
    assert max(abs(x - oracle.trim_value(x, 4, mask, 1)[0]) for x in range(256)) == 15


def test_rounding_is_floor_plus_conditional_step(oracle):
    for n, mask in all_modes():
        for x in range(256):
            f, s = oracle.trim_value(x, n, mask, 0)
            r, s2 = oracle.trim_value(x, n, mask, 1)
            assert s == s2                                   # window fixed by the unrounded value
            up = s > 0 and (x % 2 ** s) >= 2 ** (s - 1) and (f >> s) != 2 ** n - 1
            assert r == f + (2 ** s if up else 0)


def test_rounding_tie_and_saturation_readings(oracle):
    """The two readings the paper does not fix: ties go up; a carry out of the window saturates."""
    assert oracle.trim_value(27, 4, 0x1F, 1)[0] == 28        # residual 1 of 2 -> up
    assert oracle.trim_value(18, 4, 0x15, 1)[0] == 20        # residual exactly half (2 of 4) -> up
    assert oracle.trim_value(31, 4, 0x1F, 1)[0] == 30        # 15.5 -> would be 16: saturate at 15
    assert oracle.trim_value(63, 4, 0x15, 1)[0] == 60
    assert oracle.trim_value(255, 4, 0x1F, 1)[0] == 240
    assert oracle.trim_value(248, 4, 0x11, 1)[0] == 240
    assert oracle.trim_value(247, 4, 0x11, 1)[0] == 240      # 15.44 -> 15
    assert oracle.trim_value(232, 4, 0x11, 1)[0] == 240      # 14.5 -> 15 (tie up)


def test_wide_window_shift_sets(oracle):
    """A zero partner grants 2n bits: 8 (n=4), 6 (n=3), 4 (n=2) -- Section 5.1."""
    assert oracle.wide_shift_mask(4, 0x1F) == 0x01
    assert oracle.wide_shift_mask(4, 0x11) == 0x01
    assert oracle.wide_shift_mask(3, 0x3F) == 0x07           # 6-bit windows at shifts 0,1,2
    assert oracle.wide_shift_mask(2, 0x7F) == 0x1F           # 4-bit windows at shifts 0..4
    for n, mask in all_modes():
        assert oracle.wide_shift_mask(n, mask) == so.wide_options(n, mask)
    # the 4-bit window granted by 2-bit/7opt is exactly 4-bit/5opt
    for x in range(256):
        for rnd in (0, 1):
            assert oracle.trim_value(x, 4, oracle.wide_shift_mask(2, 0x7F), rnd) == \
                oracle.trim_value(x, 4, 0x1F, rnd)


@pytest.mark.parametrize("n,mask", [(4, 0x1F), (4, 0x15), (4, 0x11), (4, 0x1B), (3, 0x3F), (2, 0x7F)])
@pytest.mark.parametrize("rnd", [0, 1])
@pytest.mark.parametrize("pairing", [0, 1])
def test_all_pairs_brute_force(oracle, n, mask, rnd, pairing):
    """All 256 x 256 activation pairs through the tensor entry point vs Eq. 2 written out."""
    a, b = np.meshgrid(np.arange(256, dtype=np.uint8), np.arange(256, dtype=np.uint8), indexing="ij")
    x = np.stack([a.ravel(), b.ravel()], axis=1)             # 65536 rows of C = 2
    y = oracle.trim(x, n, mask, rnd, pairing)
    single = [so.trim(v, n, mask, rnd) for v in range(256)]
    wide_mask = so.wide_options(n, mask)
    wide = [so.trim(v, 2 * n, wide_mask, rnd) for v in range(256)] if pairing else single
    exp = np.empty_like(x)
    av, bv = x[:, 0].astype(int), x[:, 1].astype(int)
    zero_in_pair = (av == 0) | (bv == 0)
    single = np.array(single, dtype=np.uint8)
    wide = np.array(wide, dtype=np.uint8)
    exp[:, 0] = np.where(zero_in_pair & bool(pairing), wide[av], single[av])
    exp[:, 1] = np.where(zero_in_pair & bool(pairing), wide[bv], single[bv])
    assert np.array_equal(y, exp)
    if pairing and n == 4:
        assert np.array_equal(y[zero_in_pair], x[zero_in_pair])     # a pair containing a zero is unchanged
    # spot-check the scalar formulation of Eq. 2 on a few hundred pairs
    rng = np.random.default_rng(7)
    for i in rng.integers(0, 65536, 300):
        assert tuple(y[i]) == so.pair(int(av[i]), int(bv[i]), n, mask, rnd, pairing)


def test_pairs_follow_channel_parity_and_odd_tail(oracle):
    """Pairs are (c, c+1) with c even inside one row; an odd last channel pairs with an implicit zero."""
    row = np.array([[200, 0, 0, 201, 202, 203, 204]], dtype=np.uint8)     # C = 7
    y = oracle.trim(row, 4, 0x1F, 0, 1)
    assert y.tolist() == [[200, 0, 0, 201, 192, 192, 204]]
    y = oracle.trim(row, 4, 0x1F, 0, 0)                                    # -vS: everything trimmed
    assert y.tolist() == [[192, 0, 0, 192, 192, 192, 192]]
    # rows never pair across their boundary
    two = np.array([[0, 0, 77], [78, 0, 0]], dtype=np.uint8)
    assert oracle.trim(two, 4, 0x11, 0, 1).tolist() == [[0, 0, 77], [78, 0, 0]]
    # 2-bit windows: a zero partner grants four bits, not eight
    lowbit = np.array([[0, 0b10110110, 0b10110110, 3]], dtype=np.uint8)
    assert oracle.trim(lowbit, 2, 0x7F, 0, 1).tolist() == [[0, 0b10110000, 0b10000000, 3]]


def test_plain_8bit_mode_is_identity(oracle):
    x = np.arange(256, dtype=np.uint8).reshape(4, 64)
    assert np.array_equal(oracle.trim(x, 8, 0x01, 0, 0), x)


def test_tensor_trim_matches_scalar_on_random_rows(oracle):
    import sparq_synth as S
    rng = S.rng_for(9, 1)
    for C in (1, 2, 5, 16, 33):
        x = S.gen_activations((257, C), 0.5, rng)
        for n, mask in [(4, 0x1F), (4, 0x15), (3, 0x3F), (2, 0x7F)]:
            for rnd in (0, 1):
                y = oracle.trim(x, n, mask, rnd, 1)
                for r in range(0, 257, 37):
                    for c in range(0, C, 2):
                        a = int(x[r, c])
                        b = int(x[r, c + 1]) if c + 1 < C else 0
                        ea, eb = so.pair(a, b, n, mask, rnd, 1)
                        assert y[r, c] == ea
                        if c + 1 < C:
                            assert y[r, c + 1] == eb


def test_mode_validation(oracle):
    assert oracle.mode_check(4, 0x1F, 1, 1) == 0
    assert oracle.mode_check(8, 0, 0, 0) == 0
    assert oracle.mode_check(4, 0x0F, 0, 1) == 1      # bit 7 unreachable
    assert oracle.mode_check(4, 0x1E, 0, 1) == 1      # shift 0 missing
    assert oracle.mode_check(4, 0x3F, 0, 1) == 1      # window above bit 7
    assert oracle.mode_check(5, 0x0F, 0, 1) == 1
    assert oracle.mode_check(2, 0x55, 0, 0) == 0      # fine without pairing ...
    assert oracle.mode_check(2, 0x41, 0, 1) == 1      # ... but no 4-bit window reaches bit 7 here
    assert oracle.mode_check(4, 0x1F, 2, 1) == 1
    with pytest.raises(ValueError):
        oracle.trim(np.zeros((2, 2), np.uint8), 4, 0x0F, 0, 1)


def test_synthetic_activations_resemble_paper_statistics():
    """Section 5.1 reports bit 7..4 toggle rates 0.5 / 9.2 / 33.8 / 44.8 % for non-zero
    ResNet-18 activations; the half-normal stand-in must land in the same neighbourhood."""
    import sparq_synth as S
    x = S.gen_activations((1 << 20,), 0.5, S.rng_for(0, 99))
    assert abs((x == 0).mean() - 0.5) < 0.005
    nz = x[x > 0]
    rates = [float(((nz >> b) & 1).mean()) for b in (7, 6, 5, 4)]
    for got, paper, tol in zip(rates, (0.005, 0.092, 0.338, 0.448), (0.01, 0.04, 0.04, 0.05)):
        assert abs(got - paper) < tol
