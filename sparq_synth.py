"""Seeded synthetic inputs and layer tables for the SPARQ hot path.

This module holds NO arithmetic of the method (no trimming, no pairing, no
dot products): only shapes, option sets and random data.  It is the one piece
shared by the CPU oracle's tests and the GPU library's tests/benchmark, so that
both sides see identical bytes.

Data recipe (stand-in for post-ReLU ImageNet activations and trained weights,
neither of which is available offline):
  * activations: uint8, exact zeros i.i.d. with probability ``zf``; non-zeros
    ``clip(rint(|N(0,1)| * 40), 1, 255)`` -- bell-shaped magnitudes whose
    bit-7..4 toggle rates (about 0.2 / 11 / 33 / 43 %) are close to the
    0.5 / 9.2 / 33.8 / 44.8 % the paper measures on ResNet-18 (Section 5.1);
  * weights: int8 uniform in [-127, 127], layout [N][KH][KW][C];
  * scales: fp32 uniform in [1e-3, 1e-2], one per output channel;
  * numpy ``Generator(PCG64(seed))`` with seed = 20210511 + 1000*config + layer.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20210511

# window-option sets for 4-bit windows: bit t set <=> window [t+3:t] allowed
OPT5 = 0x1F
OPT3 = 0x15
OPT2 = 0x11
OPT6_3B = 0x3F   # 3-bit windows, six placements
OPT7_2B = 0x7F   # 2-bit windows, seven placements


@dataclass(frozen=True)
class Mode:
    window_bits: int = 4
    shift_mask: int = OPT5
    round_nearest: int = 1
    pair: int = 1

    def astuple(self):
        return (self.window_bits, self.shift_mask, self.round_nearest, self.pair)

    def kwargs(self):
        return dict(window_bits=self.window_bits, shift_mask=self.shift_mask,
                    round_nearest=self.round_nearest, pair=self.pair)

    @property
    def label(self) -> str:
        if self.window_bits == 8:
            return "plain8"
        nopt = bin(self.shift_mask).count("1")
        return f"{self.window_bits}b-{nopt}opt-{'round' if self.round_nearest else 'floor'}-" \
               f"{'vS' if self.pair else 'novS'}"


PLAIN8 = Mode(8, 0x01, 0, 0)


@dataclass(frozen=True)
class ConvLayer:
    name: str
    B: int
    H: int
    W: int
    C: int
    N: int
    KH: int = 1
    KW: int = 1
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (0, 0)
    zf: float = 0.5
    mode: Mode = Mode()
    repeat: int = 1          # how many identical layers of this shape the network has
    index: int = 0           # layer index used in the seed

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad[0] - self.KH) // self.stride[0] + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad[1] - self.KW) // self.stride[1] + 1

    @property
    def M(self) -> int:
        return self.B * self.Ho * self.Wo

    @property
    def K(self) -> int:
        return self.KH * self.KW * self.C

    @property
    def ops(self) -> int:
        """int8-equivalent operations (2 per multiply-accumulate)."""
        return 2 * self.M * self.K * self.N

    def x_shape(self):
        return (self.B, self.H, self.W, self.C)

    def w_shape(self):
        return (self.N, self.KH, self.KW, self.C)


# --------------------------------------------------------------------------
# random data
# --------------------------------------------------------------------------

def rng_for(config: int, layer: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + layer))


def gen_activations(shape, zf: float, rng: np.random.Generator, chunk: int = 1 << 24) -> np.ndarray:
    """uint8 ReLU-sparse half-normal activations (see module docstring)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint8)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        z = rng.standard_normal(hi - lo, dtype=np.float32)
        v = np.clip(np.rint(np.abs(z) * np.float32(40.0)), 1, 255).astype(np.uint8)
        u = rng.random(hi - lo, dtype=np.float32)
        v[u < np.float32(zf)] = 0
        out[lo:hi] = v
    return out.reshape(shape)


def gen_weights(shape, rng: np.random.Generator) -> np.ndarray:
    return rng.integers(-127, 128, size=shape, dtype=np.int8)


def gen_scales(n: int, rng: np.random.Generator) -> np.ndarray:
    return rng.uniform(1e-3, 1e-2, size=n).astype(np.float32)


def gen_requant(layer: "ConvLayer", rng: np.random.Generator) -> np.ndarray:
    """Per-output-channel requantisation factors (input scale * weight scale / output scale) sized so that the
    requantised results of the synthetic tensors use the whole unsigned 8-bit range: about half of them clamp
    at 0, a few per cent at 255 (accumulator spread ~ 2000 * sqrt(K) for these activations and weights)."""
    return (rng.uniform(0.7, 1.3, size=layer.N) * (0.044 / np.sqrt(layer.K))).astype(np.float32)


def gen_sparse24_weights(shape, rng: np.random.Generator, natural_pairs: bool = False):
    """2:4 structured-sparse int8 weights for a dense shape [N,KH,KW,C] (C a multiple of 4), in compressed form:
    (values int8 [N,KH,KW,C/2], coordinates uint8 [N,KH,KW,C/2]); of every four adjacent input channels two random
    positions are kept (ascending).  About 3 % of the kept values are zero, as a pruned-and-quantised layer has.
    natural_pairs: only the position pairs (0,1) and (2,3) are drawn."""
    N, KH, KW, C = shape
    assert C % 4 == 0
    groups = N * KH * KW * (C // 4)
    table = np.array([[0, 1], [2, 3]] if natural_pairs else [[0, 1], [0, 2], [0, 3], [1, 2], [1, 3], [2, 3]], dtype=np.uint8)
    idx = table[rng.integers(0, len(table), size=groups)]
    vals = rng.integers(-127, 128, size=(groups, 2), dtype=np.int64).astype(np.int8)
    vals[rng.random((groups, 2)) < 0.03] = 0
    return vals.reshape(N, KH, KW, C // 2), idx.reshape(N, KH, KW, C // 2)


def sparse24_to_dense(w_vals: np.ndarray, w_idx: np.ndarray) -> np.ndarray:
    """The dense [N,KH,KW,C] weights a compressed 2:4 tensor stands for (zeros at the pruned positions)."""
    N, KH, KW, C2 = w_vals.shape
    dense = np.zeros((N * KH * KW * (C2 // 2), 4), dtype=np.int8)
    v, i = w_vals.reshape(-1, 2), w_idx.reshape(-1, 2).astype(np.int64)
    r = np.arange(len(v))
    dense[r, i[:, 0]] = v[:, 0]
    dense[r, i[:, 1]] = v[:, 1]
    return dense.reshape(N, KH, KW, 2 * C2)


def gen_layer(config: int, layer: ConvLayer):
    """(x uint8 NHWC, w int8 [N,KH,KW,C], scale fp32 [N]) for one layer."""
    rng = rng_for(config, layer.index)
    x = gen_activations(layer.x_shape(), layer.zf, rng)
    w = gen_weights(layer.w_shape(), rng)
    s = gen_scales(layer.N, rng)
    return x, w, s


def _layer_zf(config: int, index: int, lo: float, hi: float) -> float:
    """Per-layer zero fraction, drawn from its own stream so tables are static."""
    r = np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + 500 + index))
    return float(r.uniform(lo, hi))


def _number(layers: List[ConvLayer]) -> List[ConvLayer]:
    return [replace(l, index=i) for i, l in enumerate(layers)]


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def config0() -> List[ConvLayer]:
    """One 3x3 conv, batch 1, 56x56x64 -> 64, 5opt round, pairing on."""
    return _number([ConvLayer("conv3x3_56x56x64_64", 1, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1), 0.5,
                              Mode(4, OPT5, 1, 1))])


def config1(batch: int = 32) -> List[ConvLayer]:
    """ResNet-18 conv layers (3opt floor, pairing on; first conv plain 8-bit)."""
    m = Mode(4, OPT3, 0, 1)
    L = [ConvLayer("conv1_7x7s2", batch, 224, 224, 3, 64, 7, 7, (2, 2), (3, 3), 0.0, PLAIN8)]
    L.append(ConvLayer("l1_3x3_64", batch, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1), mode=m, repeat=4))
    spatial, cin = 56, 64
    for stage, cout in ((2, 128), (3, 256), (4, 512)):
        L.append(ConvLayer(f"l{stage}_3x3s2_{cin}_{cout}", batch, spatial, spatial, cin, cout, 3, 3,
                           (2, 2), (1, 1), mode=m))
        L.append(ConvLayer(f"l{stage}_1x1s2_{cin}_{cout}", batch, spatial, spatial, cin, cout, 1, 1,
                           (2, 2), (0, 0), mode=m))
        spatial //= 2
        L.append(ConvLayer(f"l{stage}_3x3_{cout}", batch, spatial, spatial, cout, cout, 3, 3,
                           (1, 1), (1, 1), mode=m, repeat=3))
        cin = cout
    L = _number(L)
    return [l if l.mode.window_bits == 8 else replace(l, zf=_layer_zf(1, l.index, 0.4, 0.6)) for l in L]


def config2(batch: int = 256) -> List[ConvLayer]:
    """ResNet-50 bottleneck stack (stride on the 3x3, 5opt round, pairing on)."""
    m = Mode(4, OPT5, 1, 1)
    L = [ConvLayer("conv1_7x7s2", batch, 224, 224, 3, 64, 7, 7, (2, 2), (3, 3), 0.0, PLAIN8)]
    spatial, cin = 56, 64
    for stage, (mid, cout, blocks) in enumerate(((64, 256, 3), (128, 512, 4), (256, 1024, 6),
                                                 (512, 2048, 3)), start=1):
        s = 1 if stage == 1 else 2
        so = spatial // s
        # first block (with projection)
        L.append(ConvLayer(f"s{stage}b1_1x1_{cin}_{mid}", batch, spatial, spatial, cin, mid, mode=m))
        L.append(ConvLayer(f"s{stage}b1_3x3s{s}_{mid}", batch, spatial, spatial, mid, mid, 3, 3,
                           (s, s), (1, 1), mode=m))
        L.append(ConvLayer(f"s{stage}b1_1x1_{mid}_{cout}", batch, so, so, mid, cout, mode=m))
        L.append(ConvLayer(f"s{stage}proj_1x1s{s}_{cin}_{cout}", batch, spatial, spatial, cin, cout, 1, 1,
                           (s, s), (0, 0), mode=m))
        # remaining blocks
        r = blocks - 1
        L.append(ConvLayer(f"s{stage}bx_1x1_{cout}_{mid}", batch, so, so, cout, mid, mode=m, repeat=r))
        L.append(ConvLayer(f"s{stage}bx_3x3_{mid}", batch, so, so, mid, mid, 3, 3, (1, 1), (1, 1),
                           mode=m, repeat=r))
        L.append(ConvLayer(f"s{stage}bx_1x1_{mid}_{cout}", batch, so, so, mid, cout, mode=m, repeat=r))
        spatial, cin = so, cout
    L = _number(L)
    return [l if l.mode.window_bits == 8 else replace(l, zf=_layer_zf(2, l.index, 0.3, 0.7)) for l in L]


def config3_layer(rows: int = 65536) -> ConvLayer:
    """The large explicit GEMM: M=65536, K=4608 (3x3x512), N=512."""
    return ConvLayer("gemm_65536x4608x512", 1, rows, 1, 4608, 512, 1, 1, (1, 1), (0, 0), 0.5,
                     Mode(4, OPT5, 1, 1))


def config3_sweep():
    """36 (mode, zero fraction) points of the option sweep."""
    pts = []
    for mask in (OPT2, OPT3, OPT5):
        for rnd in (0, 1):
            for pair in (0, 1):
                for zf in (0.2, 0.5, 0.8):
                    pts.append((Mode(4, mask, rnd, pair), zf))
    return pts


def config3_sweep_low():
    """24 (mode, zero fraction) points of the lower-budget variants (Section 5.1, Table 4): 3-bit windows with
    6 shifts and 2-bit windows with 7 shifts, {floor, round} x pairing {off, on} x zero fraction {.2,.5,.8}."""
    pts = []
    for n, mask in ((3, OPT6_3B), (2, OPT7_2B)):
        for rnd in (0, 1):
            for pair in (0, 1):
                for zf in (0.2, 0.5, 0.8):
                    pts.append((Mode(n, mask, rnd, pair), zf))
    return pts


def config4(batch: int = 128, mode: Optional[Mode] = None) -> List[ConvLayer]:
    """Inception-v3-shaped mixed convolutions, 50 % zeros, incl. odd channel counts."""
    m = mode or Mode(4, OPT5, 1, 1)
    L: List[ConvLayer] = []

    def add(name, hw, c, n, kh=1, kw=1, st=(1, 1), pd=(0, 0)):
        L.append(ConvLayer(name, batch, hw, hw, c, n, kh, kw, st, pd, 0.5, m))

    # 35x35 blocks
    for c in (192, 256, 288):
        add(f"a35_1x1_{c}_64", 35, c, 64)
        add(f"a35_1x1_{c}_48", 35, c, 48)
    add("a35_1x1_288_96", 35, 288, 96)
    add("a35_5x5_48_64", 35, 48, 64, 5, 5, (1, 1), (2, 2))
    add("a35_3x3_64_96", 35, 64, 96, 3, 3, (1, 1), (1, 1))
    add("a35_3x3_96_96", 35, 96, 96, 3, 3, (1, 1), (1, 1))
    add("r35_3x3s2_288_384", 35, 288, 384, 3, 3, (2, 2), (0, 0))
    add("r35_3x3s2_96_96", 35, 96, 96, 3, 3, (2, 2), (0, 0))
    # 17x17 blocks
    for c in (128, 160, 192):
        add(f"b17_1x1_768_{c}", 17, 768, c)
        add(f"b17_1x7_{c}_{c}", 17, c, c, 1, 7, (1, 1), (0, 3))
        add(f"b17_7x1_{c}_{c}", 17, c, c, 7, 1, (1, 1), (3, 0))
    add("b17_7x1_192_192b", 17, 192, 192, 7, 1, (1, 1), (3, 0))
    add("r17_3x3s2_192_320", 17, 192, 320, 3, 3, (2, 2), (0, 0))
    add("r17_3x3s2_192_192", 17, 192, 192, 3, 3, (2, 2), (0, 0))
    # 8x8 blocks
    add("c8_1x1_768_320", 8, 768, 320)
    add("c8_1x1_768_384", 8, 768, 384)
    add("c8_1x3_384_384", 8, 384, 384, 1, 3, (1, 1), (0, 1))
    add("c8_3x1_384_384", 8, 384, 384, 3, 1, (1, 1), (1, 0))
    add("c8_3x3_448_384", 8, 448, 384, 3, 3, (1, 1), (1, 1))
    # deliberately odd channel counts (unpaired last channel, ragged K and N)
    add("odd_3x3_65_96", 35, 65, 96, 3, 3, (1, 1), (1, 1))
    add("odd_1x7_159_161", 17, 159, 161, 1, 7, (1, 1), (0, 3))
    return _number(L)


def total_ops(layers: List[ConvLayer]) -> int:
    return sum(l.ops * l.repeat for l in layers)
