"""GPU parity of the 2:4 weight-sparse path (Section 4, sparse tensor core; Section 5.3): activations picked by the
kept weights' coordinates, the picked two forming the vSPARQ pair -- int32 bit-exact against the oracle, fp32 to 1e-6."""
import numpy as np
import pytest
import torch

import sparq_synth as S

pytestmark = pytest.mark.gpu

M45 = S.Mode(4, S.OPT5, 1, 1)
LAYERS = [
    S.ConvLayer("sp_1x1_4_8", 1, 5, 7, 4, 8, 1, 1, (1, 1), (0, 0), 0.5, S.Mode(4, S.OPT5, 0, 1)),
    S.ConvLayer("sp_1x1_64_64", 2, 14, 14, 64, 64, 1, 1, (1, 1), (0, 0), 0.5, M45),
    S.ConvLayer("sp_3x3_32_48", 2, 13, 11, 32, 48, 3, 3, (1, 1), (1, 1), 0.4, M45),
    S.ConvLayer("sp_3x3s2_36_40", 2, 15, 15, 36, 40, 3, 3, (2, 2), (1, 1), 0.6, S.Mode(4, S.OPT3, 0, 1)),
    S.ConvLayer("sp_1x1_256_96", 3, 17, 17, 256, 96, 1, 1, (1, 1), (0, 0), 0.5, S.Mode(4, S.OPT2, 1, 1)),
    S.ConvLayer("sp_3x3_128_128", 2, 14, 14, 128, 128, 3, 3, (1, 1), (1, 1), 0.5, M45),
    S.ConvLayer("sp_1x7_64_32_3bit", 2, 17, 17, 64, 32, 1, 7, (1, 1), (0, 3), 0.5, S.Mode(3, S.OPT6_3B, 1, 1)),
    S.ConvLayer("sp_3x3_64_64_2bit", 2, 9, 9, 64, 64, 3, 3, (1, 1), (1, 1), 0.5, S.Mode(2, S.OPT7_2B, 0, 1)),
    S.ConvLayer("sp_3x3_64_64_novS", 2, 9, 9, 64, 64, 3, 3, (1, 1), (1, 1), 0.5, S.Mode(4, S.OPT5, 1, 0)),
    S.ConvLayer("sp_1x1_68_20_novS", 2, 9, 9, 68, 20, 1, 1, (1, 1), (0, 0), 0.5, S.Mode(4, S.OPT3, 0, 0)),
    S.ConvLayer("sp_3x3_64_64_plain8", 2, 9, 9, 64, 64, 3, 3, (1, 1), (1, 1), 0.5, S.PLAIN8),
]


# shapes for the sparse matrix instruction's kernel: ragged pixel and channel tiles, channel counts that are not a
# multiple of 4 (scalar result stores), strides, wide layers (256-channel tiles), long reductions
SPARSE_MFMA_LAYERS = [
    S.ConvLayer("spm_3x3_64_50", 2, 13, 11, 64, 50, 3, 3, (1, 1), (1, 1), 0.5, M45),
    S.ConvLayer("spm_3x3_32_300", 3, 12, 12, 32, 300, 3, 3, (1, 1), (1, 1), 0.4, M45),
    S.ConvLayer("spm_1x1s2_64_130", 2, 15, 15, 64, 130, 1, 1, (2, 2), (0, 0), 0.5, M45),
    S.ConvLayer("spm_3x3s2_48_72", 2, 17, 17, 48, 72, 3, 3, (2, 2), (1, 1), 0.6, S.Mode(4, S.OPT3, 0, 1)),
    S.ConvLayer("spm_5x5_16_33", 1, 20, 20, 16, 33, 5, 5, (1, 1), (2, 2), 0.5, S.Mode(3, S.OPT6_3B, 1, 1)),
    S.ConvLayer("spm_1x1_512_256", 1, 23, 23, 512, 256, 1, 1, (1, 1), (0, 0), 0.5, M45),
    S.ConvLayer("spm_3x3_128_64_plain8", 2, 19, 19, 128, 64, 3, 3, (1, 1), (1, 1), 0.5, S.PLAIN8),
    S.ConvLayer("spm_1x1_96_64", 2, 15, 15, 96, 64, 1, 1, (1, 1), (0, 0), 0.5, M45),
    S.ConvLayer("spm_3x3_64_72_novS_round4", 2, 17, 15, 64, 72, 3, 3, (1, 1), (1, 1), 0.5, S.Mode(4, S.OPT5, 1, 0)),
    S.ConvLayer("spm_3x3s2_128_50_novS_floor", 2, 17, 17, 128, 50, 3, 3, (2, 2), (1, 1), 0.4, S.Mode(4, S.OPT3, 0, 0)),
    S.ConvLayer("spm_1x1_256_260_novS_round3", 2, 15, 15, 256, 260, 1, 1, (1, 1), (0, 0), 0.5, S.Mode(3, S.OPT6_3B, 1, 0)),
    S.ConvLayer("spm_1x7_64_64_novS_floor2", 2, 17, 17, 64, 64, 1, 7, (1, 1), (0, 3), 0.5, S.Mode(2, S.OPT7_2B, 0, 0)),
    S.ConvLayer("spm_1x1_192_100_plain8", 2, 19, 19, 192, 100, 1, 1, (1, 1), (0, 0), 0.5, S.PLAIN8),
]
FORMS = [None, "path=gather", "path=patch,patch_ws=1", "path=patch,patch_ws=1,patch_tn=64", "path=patch,patch_ws=1,patch_tn=128",
         "path=patch,patch_ws=1,patch_tn=256"]


@pytest.fixture(scope="module")
def sq():
    assert torch.cuda.is_available(), "GPU tests need a device"
    import paper_2105_11010_amd as sq_
    return sq_


def run_sparse(sq, layer, x, wv, wi, sc):
    dev = torch.device("cuda:0")
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    m = sq.mode(*layer.mode.astuple())
    xd, vd, idd, sd = (torch.from_numpy(a).to(dev) for a in (x, wv, wi, sc))
    packed = torch.empty(sq.sparq_sparse24_packed_bytes(d, m), dtype=torch.uint8, device=dev)
    sq.sparq_pack_weights_sparse24(vd, idd, d, m, packed)
    wsb = sq.sparq_sparse24_workspace_bytes(d, m)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev) if wsb else None
    acc = torch.empty((layer.M, layer.N), dtype=torch.int32, device=dev)
    out = torch.empty((layer.M, layer.N), dtype=torch.float32, device=dev)
    sq.sparq_conv_gemm_sparse24(xd, packed, d, m, acc=acc, scale=sd, out=out, workspace=ws)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), out.cpu().numpy()


@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: l.name)
def test_sparse24_convolution(sq, oracle, layer):
    rng = S.rng_for(10, LAYERS.index(layer))
    x = S.gen_activations(layer.x_shape(), layer.zf, rng)
    wv, wi = S.gen_sparse24_weights(layer.w_shape(), rng)
    sc = S.gen_scales(layer.N, rng)
    acc, out = run_sparse(sq, layer, x, wv, wi, sc)
    ref_acc, ref_out = oracle.conv_gemm_sparse24(x, wv, wi, layer.stride, layer.pad, scale=sc, **layer.mode.kwargs())
    assert np.array_equal(acc, ref_acc), f"{layer.name}: int32 accumulators differ from the oracle"
    assert np.all(np.abs(out.astype(np.float64) - ref_out) <= 1e-6 * np.abs(ref_out))


@pytest.mark.parametrize("layer", SPARSE_MFMA_LAYERS, ids=lambda l: l.name)
def test_sparse24_on_the_sparse_matrix_instruction(sq, oracle, layer):
    """Every kernel form the layer can take (the rules' choice, the gather kernel, the wave-specialised input-patch
    kernel at each tile width) against the oracle; the patch forms must report the sparse matrix instruction."""
    rng = S.rng_for(10, 100 + SPARSE_MFMA_LAYERS.index(layer))
    x = S.gen_activations(layer.x_shape(), layer.zf, rng)
    wv, wi = S.gen_sparse24_weights(layer.w_shape(), rng)
    sc = S.gen_scales(layer.N, rng)
    ref_acc, ref_out = oracle.conv_gemm_sparse24(x, wv, wi, layer.stride, layer.pad, scale=sc, **layer.mode.kwargs())
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    m = sq.mode(*layer.mode.astuple())
    seen = set()
    try:
        for spec in FORMS:
            sq.sparq_set_tuning(spec)
            plan = sq.sparq_sparse24_plan(d, m)
            if spec and "patch" in spec:
                assert "conv_patch_kernel" not in plan or plan.endswith("sparse_mfma"), plan
            if spec == "path=gather":
                assert plan.endswith("dense_mfma"), plan
            seen.add(plan)
            acc, out = run_sparse(sq, layer, x, wv, wi, sc)
            assert np.array_equal(acc, ref_acc), f"{layer.name} [{plan}]: int32 accumulators differ from the oracle"
            assert np.all(np.abs(out.astype(np.float64) - ref_out) <= 1e-6 * np.abs(ref_out)), plan
    finally:
        sq.sparq_set_tuning(None)
    assert any(p.endswith("sparse_mfma") for p in seen), seen


@pytest.mark.parametrize("layer", [SPARSE_MFMA_LAYERS[0], SPARSE_MFMA_LAYERS[5]], ids=lambda l: l.name)
def test_sparse_instruction_kernel_with_one_output(sq, oracle, layer):
    """int32 accumulators alone and fp32 results alone (each its own copy of the epilogue)."""
    rng = S.rng_for(10, 200 + SPARSE_MFMA_LAYERS.index(layer))
    x = S.gen_activations(layer.x_shape(), layer.zf, rng)
    wv, wi = S.gen_sparse24_weights(layer.w_shape(), rng)
    sc = S.gen_scales(layer.N, rng)
    ref_acc, ref_out = oracle.conv_gemm_sparse24(x, wv, wi, layer.stride, layer.pad, scale=sc, **layer.mode.kwargs())
    dev = torch.device("cuda:0")
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    m = sq.mode(*layer.mode.astuple())
    assert sq.sparq_sparse24_plan(d, m).endswith("sparse_mfma")
    xd, vd, idd, sd = (torch.from_numpy(a).to(dev) for a in (x, wv, wi, sc))
    packed = torch.empty(sq.sparq_sparse24_packed_bytes(d, m), dtype=torch.uint8, device=dev)
    sq.sparq_pack_weights_sparse24(vd, idd, d, m, packed)
    ws = torch.empty(max(sq.sparq_sparse24_workspace_bytes(d, m), 1), dtype=torch.uint8, device=dev)
    acc = torch.full((layer.M, layer.N), -7, dtype=torch.int32, device=dev)
    out = torch.full((layer.M, layer.N), -7.0, dtype=torch.float32, device=dev)
    sq.sparq_conv_gemm_sparse24(xd, packed, d, m, acc=acc, workspace=ws)
    sq.sparq_conv_gemm_sparse24(xd, packed, d, m, scale=sd, out=out, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref_acc)
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - ref_out) <= 1e-6 * np.abs(ref_out))


def test_extreme_values(sq, oracle):
    """All activations 255 or 0 in a pattern that makes every partner case occur, weights at -127 / 127."""
    layer = S.ConvLayer("sp_extreme", 1, 6, 6, 64, 32, 3, 3, (1, 1), (1, 1), 0.5, M45)
    rng = S.rng_for(10, 50)
    x = (rng.integers(0, 2, layer.x_shape()) * 255).astype(np.uint8)
    wv, wi = S.gen_sparse24_weights(layer.w_shape(), rng)
    wv = np.where(wv >= 0, 127, -127).astype(np.int8)
    sc = S.gen_scales(layer.N, rng)
    acc, _ = run_sparse(sq, layer, x, wv, wi, sc)
    ref_acc, _ = oracle.conv_gemm_sparse24(x, wv, wi, layer.stride, layer.pad, **layer.mode.kwargs())
    assert np.array_equal(acc, ref_acc)


def test_rejections(sq):
    m = sq.mode(4, S.OPT5, 1, 1)
    assert sq.sparq_sparse24_packed_bytes(sq.conv_desc(1, 4, 4, 6, 8), m) == 0          # C not a multiple of 4
    d = sq.conv_desc(1, 4, 4, 8, 8)
    x = torch.zeros((1, 4, 4, 8), dtype=torch.uint8, device="cuda")
    packed = torch.zeros(sq.sparq_sparse24_packed_bytes(d, m), dtype=torch.uint8, device="cuda")
    out = torch.zeros((16, 8), dtype=torch.float32, device="cuda")
    sc = torch.ones(8, dtype=torch.float32, device="cuda")
    with pytest.raises(sq.SparqError) as e:
        sq.sparq_conv_gemm_sparse24(x, packed, d, m, scale=sc, out=out, workspace=torch.zeros(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3                                                          # workspace too small
