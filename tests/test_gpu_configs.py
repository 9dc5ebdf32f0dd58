"""GPU parity at the benchmark's full sizes: every layer of the five workload tables runs through
the C ABI exactly as bench.py launches it (full tensors, fused dequantisation); the CPU oracle then
recomputes a sample of output rows one by one -- first and last tile, image borders, random interior
rows; 4096 and more rows on the largest layers -- and those must match bit-exactly (int32, and the
requantised uint8 bytes of the second entry point) and to 1e-6 relative (fp32)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import sparq_synth as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sq():
    assert torch.cuda.is_available(), "GPU tests need a device"
    import paper_2105_11010_amd as sq_
    return sq_


def sample_rows(layer, n=160, seed=0):
    """Output rows to recompute: tile edges, image borders, and a random remainder."""
    M, Ho, Wo = layer.M, layer.Ho, layer.Wo
    rows = {0, 1, 127, 128, 129, M - 1, M - 2, M - 128, M - 129, M // 2}
    for b in (0, layer.B - 1):
        base = b * Ho * Wo
        for oy in (0, Ho - 1, Ho // 2):
            for ox in (0, Wo - 1, Wo // 3):
                rows.add(base + oy * Wo + ox)
    rng = np.random.default_rng(1234 + seed)
    rows.update(int(r) for r in rng.integers(0, M, size=n))
    return np.array(sorted(r for r in rows if 0 <= r < M), dtype=np.int64)


def check_sampled(sq, oracle, cfg_id, layer, n=160, modes=None, full=False):
    """Run `layer` at full size under each mode (default: the layer's own) on one set of tensors.
    full: the oracle recomputes EVERY output row, not a sample."""
    data = S.gen_layer(cfg_id, layer)
    for mode in modes or [layer.mode]:
        _check_one(sq, oracle, replace(layer, mode=mode), data, n, full)


_PLANS = {}


def bench_plans(sq, workload):
    if workload not in _PLANS:
        _PLANS[workload] = _bench_plans(sq, workload)
    return _PLANS[workload]


def _bench_plans(sq, workload):
    """{layer name: plan line} of what `bench.py --workload <workload>` launches (its own layer list, batch and modes)."""
    import argparse

    import bench
    args = argparse.Namespace(workload=workload, rows=65536, batch=None, mask=None, round=None, pair=None, zf=None)
    _, layers, _ = bench.build_workload(args)
    plans = {}
    for l in layers:
        d = sq.conv_desc(l.B, l.H, l.W, l.C, l.N, l.KH, l.KW, l.stride, l.pad)
        plans[l.name] = sq.sparq_conv_plan(d, sq.mode(*l.mode.astuple()))
    return plans


def assert_plan_is_the_benchmarks(sq, workload, layer):
    """The kernel and tiling this test runs for `layer` are the ones the benchmark times for it."""
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    mine = sq.sparq_conv_plan(d, sq.mode(*layer.mode.astuple()))
    assert mine == bench_plans(sq, workload)[layer.name], f"{layer.name}: tested {mine!r}, benchmark launches another plan"


def _check_one(sq, oracle, layer, data, n, full=False):
    x, w, sc = data
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    m = sq.mode(*layer.mode.astuple())
    dev = torch.device("cuda:0")
    xd, wd, sd = (torch.from_numpy(a).to(dev) for a in (x, w, sc))
    packed = torch.empty(sq.sparq_packed_bytes(d), dtype=torch.uint8, device=dev)
    sq.sparq_pack_weights(wd, d, packed)
    wsb = sq.sparq_workspace_bytes(d, m)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev) if wsb else None
    acc = torch.empty((layer.M, layer.N), dtype=torch.int32, device=dev)
    out = torch.empty((layer.M, layer.N), dtype=torch.float32, device=dev)
    sq.sparq_conv_gemm(xd, packed, d, m, acc=acc, scale=sd, out=out, workspace=ws)
    rows = None if full else sample_rows(layer, n, seed=layer.index)
    ridx = torch.from_numpy(rows).to(dev) if rows is not None else slice(None)
    got_acc = acc[ridx].cpu().numpy()
    got_out = out[ridx].cpu().numpy()
    # a property that holds at any size: the fused fp32 output is the dequantised accumulator
    deq = torch.empty_like(out)
    sq.sparq_dequant(acc, sd, deq)
    assert torch.equal(deq, out), f"{layer.name}: fused and standalone dequantisation differ"
    del out, deq
    # the requantised-output entry point on the same tensors: its bytes are the requantised accumulators
    # everywhere (a property at any size), and equal the oracle's on the sampled rows
    fq = S.gen_requant(layer, S.rng_for(2, 900 + layer.index))
    fd = torch.from_numpy(fq).to(dev)
    y = torch.empty((layer.M, layer.N), dtype=torch.uint8, device=dev)
    sq.sparq_conv_gemm_u8(xd, packed, d, m, fd, y, workspace=ws)
    y2 = torch.empty_like(y)
    sq.sparq_requant(acc, fd, y2)
    assert torch.equal(y, y2), f"{layer.name}: fused and standalone requantisation differ"
    got_y = y[ridx].cpu().numpy()
    torch.cuda.synchronize()
    del acc, y, y2, xd
    ref_acc, ref_out = oracle.conv_gemm(x, w, layer.stride, layer.pad, scale=sc, rows=rows, **layer.mode.kwargs())
    assert int(got_acc.astype(np.int64).sum()) == int(ref_acc.astype(np.int64).sum()), f"{layer.name}: checksum of sampled rows"
    assert np.array_equal(got_acc, ref_acc), f"{layer.name} {layer.mode.label}: int32 mismatch on sampled rows"
    assert np.all(np.abs(got_out.astype(np.float64) - ref_out) <= 1e-6 * np.abs(ref_out)), f"{layer.name}: fp32 off"
    assert np.array_equal(got_y, oracle.requant(ref_acc, fq)), f"{layer.name} {layer.mode.label}: uint8 mismatch on sampled rows"


# ---- config 0: the single 3x3 convolution, every output compared ----------------------------------
def test_config0_every_output(sq, oracle):
    layer = S.config0()[0]
    assert_plan_is_the_benchmarks(sq, "cfg0", layer)
    check_sampled(sq, oracle, 0, layer, full=True)


# ---- config 1: ResNet-18, batch 32, 3opt floor (first conv plain 8-bit): every output compared ----
@pytest.mark.parametrize("layer", S.config1(), ids=lambda l: l.name)
def test_config1_resnet18_every_output(sq, oracle, layer):
    assert_plan_is_the_benchmarks(sq, "cfg1", layer)
    check_sampled(sq, oracle, 1, layer, full=True)


# ---- config 2: ResNet-50, batch 256, 5opt round: all 29 layer shapes at the stated batch -----------
@pytest.mark.parametrize("layer", S.config2(), ids=lambda l: l.name)
def test_config2_resnet50_batch_256(sq, oracle, layer):
    """Every layer at batch 256 (input up to 205 MB, fp32 output up to 822 MB), with the kernel and tiling the
    benchmark launches for it; the oracle recomputes 4096 and more sampled rows."""
    assert layer.B == 256
    assert_plan_is_the_benchmarks(sq, "cfg2", layer)
    check_sampled(sq, oracle, 2, layer, n=4096)


# ---- config 3: the option sweep on M=65536, K=4608, N=512 ------------------------------------------
@pytest.mark.parametrize("zf,modes", [(0.5, [S.Mode(4, S.OPT5, 0, 0)]),
                                      (0.2, [S.Mode(4, S.OPT3, 0, 1)]),
                                      (0.8, [S.Mode(4, S.OPT2, 1, 0)])], ids=["zf0.5", "zf0.2", "zf0.8"])
def test_config3_full_size(sq, oracle, zf, modes):
    check_sampled(sq, oracle, 3, replace(S.config3_layer(), zf=zf), n=4096, modes=modes)


def test_config3_full_size_every_output(sq, oracle):
    """The materialised A[M,K] form at the benchmark's mode: all 65536 x 512 results against the oracle."""
    layer = S.config3_layer()
    assert_plan_is_the_benchmarks(sq, "cfg3", layer)
    check_sampled(sq, oracle, 3, layer, full=True)


def test_config3_full_size_as_convolution_every_output(sq, oracle):
    """The same M, K, N as a 3x3 convolution over 512 channels (the benchmark's default workload): all
    65536 x 512 results against the oracle."""
    layer = replace(S.config3_layer(), name="conv3x3_512_512_32x32", B=64, H=32, W=32, C=512, KH=3, KW=3, pad=(1, 1))
    assert_plan_is_the_benchmarks(sq, "cfg3-conv", layer)
    check_sampled(sq, oracle, 3, layer, full=True)


@pytest.mark.parametrize("mode,zf", S.config3_sweep(), ids=lambda v: v.label if isinstance(v, S.Mode) else f"zf{v}")
def test_config3_sweep_all_36_points_small_m(sq, oracle, mode, zf):
    check_sampled(sq, oracle, 3, replace(S.config3_layer(1024 + 77), mode=mode, zf=zf), n=48)


@pytest.mark.parametrize("mode,zf", S.config3_sweep_low(), ids=lambda v: v.label if isinstance(v, S.Mode) else f"zf{v}")
def test_config3_low_bit_sweep_all_24_points_small_m(sq, oracle, mode, zf):
    """3-bit / 6-shift and 2-bit / 7-shift windows, with and without pairing (a zero partner grants 6 / 4 bits)."""
    check_sampled(sq, oracle, 3, replace(S.config3_layer(1024 + 77), mode=mode, zf=zf), n=48)


def test_config3_full_size_as_convolution_low_bit(sq, oracle):
    layer = replace(S.config3_layer(), name="conv3x3_512_512_32x32", B=64, H=32, W=32, C=512, KH=3, KW=3, pad=(1, 1))
    check_sampled(sq, oracle, 3, layer, n=2048, modes=[S.Mode(3, S.OPT6_3B, 1, 1), S.Mode(2, S.OPT7_2B, 0, 0)])


# ---- config 4: Inception-v3-shaped layers, batch 128, 4-bit 5opt and 2-bit 7opt ---------------------
@pytest.mark.parametrize("layer", S.config4(), ids=lambda l: l.name)
def test_config4_inception_4bit_and_2bit(sq, oracle, layer):
    """Both passes of the workload on the same tensors: 4-bit 5opt rounding, then the 2-bit window
    with 7 shifts where a zero partner grants 4 bits."""
    assert_plan_is_the_benchmarks(sq, "cfg4", layer)
    check_sampled(sq, oracle, 4, layer, n=512, modes=[layer.mode, S.Mode(2, S.OPT7_2B, 1, 1)])


# ---- sizes at the limits of the index arithmetic ------------------------------------------------------
def _big_1x1(sq, oracle, pixels, C, N, seed):
    """A 1x1 layer over `pixels` pixels whose activations repeat a seeded 32 MiB block (fast to generate)."""
    layer = S.ConvLayer(f"big_{pixels}x{C}x{N}", 1, pixels, 1, C, N)
    rng = S.rng_for(5, seed)
    block = S.gen_activations((1 << 25,), 0.5, rng)
    x = np.resize(block, layer.x_shape())
    w = S.gen_weights(layer.w_shape(), rng)
    sc = S.gen_scales(N, rng)
    _check_one(sq, oracle, layer, (x, w, sc), 512)


def test_patch_kernel_at_its_largest_row_count(sq, oracle):
    """M = 2^22 - 5: the last M the reciprocal divisions of the input-patch kernel accept, with a ragged last tile."""
    d = sq.conv_desc(1, (1 << 22) - 5, 1, 64, 64, 1, 1, (1, 1), (0, 0))
    assert "conv_patch_kernel" in sq.sparq_conv_plan(d, sq.mode(4, S.OPT5, 1, 1))
    _big_1x1(sq, oracle, (1 << 22) - 5, 64, 64, 1)


def test_row_count_past_the_patch_kernel_limit_takes_the_gather_kernel(sq, oracle):
    d = sq.conv_desc(1, (1 << 22) + 3, 1, 64, 64, 1, 1, (1, 1), (0, 0))
    assert "conv_gemm_kernel" in sq.sparq_conv_plan(d, sq.mode(4, S.OPT5, 1, 1))
    _big_1x1(sq, oracle, (1 << 22) + 3, 64, 64, 2)


def test_input_just_below_two_gib(sq, oracle):
    """x of 2^31 - 64 * 7 bytes (offsets are 32-bit with the top bit marking padding); outputs of 2 GiB each."""
    _big_1x1(sq, oracle, (1 << 25) - 7, 64, 16, 3)


def test_input_of_two_gib_is_refused(sq):
    d = sq.conv_desc(1, 1 << 25, 1, 64, 16, 1, 1, (1, 1), (0, 0))
    m = sq.mode(4, S.OPT5, 1, 1)
    packed = torch.empty(sq.sparq_packed_bytes(d), dtype=torch.uint8, device="cuda:0")
    x = torch.empty(1 << 31, dtype=torch.uint8, device="cuda:0")
    out = torch.empty(((1 << 25), 16), dtype=torch.float32, device="cuda:0")
    sc = torch.ones(16, dtype=torch.float32, device="cuda:0")
    with pytest.raises(sq.SparqError):
        sq.sparq_conv_gemm(x, packed, d, m, scale=sc, out=out)

