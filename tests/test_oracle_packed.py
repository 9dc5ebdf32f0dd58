"""Pins of the oracle's packed storage of trimmed activations (CPU only).

The paper fixes the fields: an n-bit window with an identifier of its position (Section 3.1: 3 bits for the five
placements of 5opt), "2-bit ShiftCtrl and 1-bit MuxCtrl" per 4-bit datum for 3opt (Section 5.1), and the multiplier
that consumes them, 2^opt1 * x1 * w1 + 2^opt2 * x2 * w2 with multiplexers choosing the weight (Eq. 4).  The tests tie
the oracle's encoder and decoder to those: bit budgets, hand-worked records, a field parser written here (not the
oracle's) fed through Eq. 4 for every pair of values, and the round trip against the trim itself."""
import itertools

import numpy as np
import pytest

import sparq_synth as S

MODES4 = [(4, m, r, p) for m in (S.OPT5, S.OPT3, S.OPT2) for r in (0, 1) for p in (0, 1)]
MODES_LOW = [(3, S.OPT6_3B, r, p) for r in (0, 1) for p in (0, 1)] + [(2, S.OPT7_2B, r, p) for r in (0, 1) for p in (0, 1)]


def kw(mode):
    n, m, r, p = mode
    return dict(window_bits=n, shift_mask=m, round_nearest=r, pair=p)


def all_pairs():
    a, b = np.meshgrid(np.arange(256), np.arange(256), indexing="ij")
    return np.stack([a.ravel(), b.ravel()], axis=1).astype(np.uint8).reshape(-1, 32)   # rows of 16 pairs


def parse_record(rec, n, mask, pair, group=1):
    """Fields of one record, decoded HERE from the layout the header documents: lists q[32], shift[32], mux[32]."""
    bits = np.unpackbits(np.frombuffer(bytes(rec), dtype=np.uint8), bitorder="little")
    shifts_allowed = [t for t in range(8) if (mask >> t) & 1]
    sb = max(1, int(np.ceil(np.log2(len(shifts_allowed)))))
    field = lambda base, k, w: int(sum(int(bits[base + k * w + i]) << i for i in range(w)))
    data0, shift0 = 0, 32 * n
    mux0 = shift0 + 32 * ((32 // group * sb + 31) // 32)
    q = [field(data0, k, n) for k in range(32)]
    sh = [shifts_allowed[field(shift0, k // group, sb)] for k in range(32)]
    mx = [int(bits[mux0 + k]) if pair else k & 1 for k in range(32)]
    return q, sh, mx


@pytest.mark.parametrize("n,mask,pair,bits_per_activation", [
    (4, S.OPT5, 0, 4 + 3),        # Section 3.1: the 4-bit window "is accompanied by a 3-bit identifier"
    (4, S.OPT3, 1, 4 + 2 + 1),    # Section 5.1: "2-bit ShiftCtrl and 1-bit MuxCtrl" per 4-bit datum
    (4, S.OPT5, 1, 4 + 3 + 1), (4, S.OPT3, 0, 4 + 2), (4, S.OPT2, 0, 4 + 1), (4, S.OPT2, 1, 4 + 1 + 1),
    (3, S.OPT6_3B, 1, 3 + 3 + 1), (2, S.OPT7_2B, 1, 2 + 3 + 1), (2, S.OPT7_2B, 0, 2 + 3)])
def test_bit_budget_per_activation(oracle, n, mask, pair, bits_per_activation):
    assert oracle.packed_record_bytes(window_bits=n, shift_mask=mask, round_nearest=0, pair=pair) * 8 == 32 * bits_per_activation


def test_what_cannot_be_packed(oracle):
    assert oracle.packed_record_bytes(window_bits=8, shift_mask=1, round_nearest=0, pair=0) == 0       # plain 8-bit layer
    assert oracle.packed_record_bytes(3, window_bits=4, shift_mask=S.OPT5, round_nearest=0, pair=0) == 0  # 3 does not divide 32
    assert oracle.packed_record_bytes(4, window_bits=4, shift_mask=S.OPT5, round_nearest=0, pair=1) == 0  # shared shift with vSPARQ
    assert oracle.packed_record_bytes(window_bits=4, shift_mask=0x0E, round_nearest=0, pair=0) == 0     # invalid option set
    with pytest.raises(ValueError):
        oracle.pack_act(np.zeros((1, 32), np.uint8), window_bits=8, shift_mask=1, round_nearest=0, pair=0)


def test_hand_worked_record_5opt_without_pairing(oracle):
    """27 = 00011011b -> window [4:1] = 1101b at shift 1 (the paper's example, Section 3.1); 3 -> 0011b at shift 0;
    200 = 11001000b -> 1100b at shift 4; 33 -> 1000b at shift 2 (Section 3.1, piecewise-linear paragraph)."""
    x = np.zeros((1, 32), np.uint8)
    x[0, :4] = [27, 3, 200, 33]
    rec = oracle.pack_act(x, window_bits=4, shift_mask=S.OPT5, round_nearest=0, pair=0)[0]
    assert len(rec) == 28
    assert list(rec[:2]) == [0b0011_1101, 0b1000_1100] and not rec[2:16].any()                 # nibbles 13,3 | 12,8
    # ShiftCtrl, 3 bits each, shifts 1,0,4,2 (5opt: code = shift): 001 | 000<<3 | 100<<6 | 010<<9 = 0x501
    assert list(rec[16:18]) == [0x01, 0x05] and not rec[18:].any()


def test_hand_worked_record_3opt_with_pairing(oracle):
    """Pairs (27,3): both non-zero -> 27 at [5:2] = 0110b (Section 3.1: 3opt places it there), 3 at [3:0];
    (27,0): zero partner -> 27 keeps 8 bits as halves 0001b << 4 and 1011b << 0, both for channel 0 of the pair;
    (0,200): halves 1100b << 4, 1000b << 0, both for channel 1; the all-zero pairs that fill the record fall under
    the first case of Eq. 2 (second value zero): halves 0 << 4 and 0 << 0 for channel 0."""
    x = np.zeros((1, 32), np.uint8)
    x[0, :6] = [27, 3, 27, 0, 0, 200]
    rec = oracle.pack_act(x, window_bits=4, shift_mask=S.OPT3, round_nearest=0, pair=1)[0]
    assert len(rec) == 28
    assert list(rec[:3]) == [0b0011_0110, 0b1011_0001, 0b1000_1100] and not rec[3:16].any()
    # ShiftCtrl 2 bits, codes of shifts {0,2,4} = {0,1,2}: data shifts 2,0 | 4,0 | 4,0 | 4,0 ... -> 01,00,10,00 | 10,00,10,00 ...
    assert rec[16] == 0b00_10_00_01 and all(b == 0b00_10_00_10 for b in rec[17:24])
    # MuxCtrl: datum -> channel of its pair: 0,1 | 0,0 | 1,1 | 0,0 ...
    assert int.from_bytes(bytes(rec[24:28]), "little") == 0b11_00_10
    assert list(oracle.unpack_act(rec[None], (1, 32), window_bits=4, shift_mask=S.OPT3, round_nearest=0, pair=1)[0, :6]) == [24, 3, 27, 0, 0, 200]


@pytest.mark.parametrize("mode", MODES4 + MODES_LOW, ids=str)
def test_round_trip_is_the_trim_on_every_pair(oracle, mode):
    x = all_pairs()
    packed = oracle.pack_act(x, **kw(mode))
    assert np.array_equal(oracle.unpack_act(packed, x.shape, **kw(mode)), oracle.trim(x, **kw(mode)))


@pytest.mark.parametrize("mode", MODES4 + MODES_LOW, ids=str)
def test_fields_fed_through_the_multiplier_of_eq4(oracle, mode):
    """For every pair (a, b): sum over its two data of 2^opt * x * w[MuxCtrl] equals T(a) * w_a + T(b) * w_b, the
    fields read by the parser of this file; every datum fits n bits and every shift is an allowed placement."""
    n, mask, r, p = mode
    rng = np.random.default_rng(5)
    rows = rng.choice(65536 // 16, size=160, replace=False)
    x = all_pairs()[rows]
    x[:, 0:2] = [[0, 0]]                                       # make sure the both-zero pair is in every row
    packed = oracle.pack_act(x, **kw(mode))
    t = oracle.trim(x, **kw(mode)).astype(np.int64)
    w = rng.integers(-127, 128, size=(len(rows), 32))
    for i in range(len(rows)):
        q, sh, mx = parse_record(packed[i], n, mask, p)
        assert max(q) < (1 << n) and all((mask >> s) & 1 for s in sh)
        for j in range(0, 32, 2):
            got = sum((q[k] << sh[k]) * int(w[i, j + (mx[k] if p else k - j)]) for k in (j, j + 1))
            assert got == int(t[i, j] * w[i, j] + t[i, j + 1] * w[i, j + 1]), (mode, x[i, j:j + 2])


def test_channel_counts_that_do_not_fill_a_record(oracle):
    rng = S.rng_for(6, 1)
    for C in (1, 3, 31, 33, 65, 100):
        x = S.gen_activations((7, C), 0.4, rng)
        for mode in ((4, S.OPT5, 1, 1), (4, S.OPT3, 0, 0), (2, S.OPT7_2B, 1, 1)):
            packed = oracle.pack_act(x, **kw(mode))
            assert packed.shape == (7, (C + 31) // 32 * oracle.packed_record_bytes(**kw(mode)))
            assert np.array_equal(oracle.unpack_act(packed, x.shape, **kw(mode)), oracle.trim(x, **kw(mode)))


@pytest.mark.parametrize("group", [2, 4, 8, 16, 32])
@pytest.mark.parametrize("mode", [(4, S.OPT5, 0, 0), (4, S.OPT5, 1, 0), (4, S.OPT3, 1, 0), (3, S.OPT6_3B, 0, 0)], ids=str)
def test_shared_shift_groups(oracle, group, mode):
    """Section 6, ShiftCtrl shared by a group (a reading; vSPARQ off): the shift is the one bSPARQ gives the group's
    largest value; every value is a multiple of 2^shift below 2^n * 2^shift, off by less than 2^shift (by at most
    half of it when rounding does not saturate), and the largest value itself decodes to its own trim under floor."""
    n, mask, r, _ = mode
    rng = S.rng_for(6, group)
    x = S.gen_activations((500, 64), 0.5, rng)
    x[0, :group] = 0                                           # an all-zero group
    x[1, :group] = 255
    packed = oracle.pack_act(x, group, **kw(mode))
    sb = int(np.ceil(np.log2(bin(mask).count("1"))))
    assert packed.shape[1] == 2 * 4 * (n + (32 // group * sb + 31) // 32)
    y = oracle.unpack_act(packed, x.shape, group, **kw(mode)).astype(int)
    xg, yg = x.reshape(500, -1, group).astype(int), y.reshape(500, -1, group)
    for i, g in itertools.product(range(500), range(64 // group)):
        top = xg[i, g].max()
        s = oracle.trim_value(top, n, mask, 0)[1]
        assert np.all(yg[i, g] % (1 << s) == 0) and np.all(yg[i, g] >> s < (1 << n))
        err = np.abs(yg[i, g] - xg[i, g])
        assert np.all(err < (1 << s))
        if r:
            unsat = (yg[i, g] >> s) < (1 << n) - 1
            assert np.all(err[unsat] * 2 <= (1 << s))
        else:
            assert yg[i, g].max() == oracle.trim_value(top, n, mask, 0)[0]
            assert np.all(yg[i, g] == (xg[i, g] >> s) << s)
    if group == 1:
        assert np.array_equal(y, oracle.trim(x, **kw(mode)))


def test_group_of_one_is_the_per_value_format(oracle):
    x = all_pairs()[:512]
    for mode in ((4, S.OPT5, 1, 0), (4, S.OPT2, 0, 0)):
        assert np.array_equal(oracle.pack_act(x, 1, **kw(mode)), oracle.pack_act(x, **kw(mode)))
