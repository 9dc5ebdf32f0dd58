"""GPU parity of the packed activation storage (Sections 3.1, 5.1, 6; Eq. 4): records bit-exact against the oracle's,
unpacked values against the oracle's, the round trip against the trim, and the convolution that reads packed input."""
import numpy as np
import pytest
import torch

import sparq_synth as S

pytestmark = pytest.mark.gpu

MODES = [(4, m, r, p) for m in (S.OPT5, S.OPT3, S.OPT2) for r in (0, 1) for p in (0, 1)] + \
        [(3, S.OPT6_3B, r, p) for r in (0, 1) for p in (0, 1)] + [(2, S.OPT7_2B, r, p) for r in (0, 1) for p in (0, 1)] + \
        [(4, 0x17, 1, 1), (3, 0x2B, 0, 0)]          # option sets of four placements: 2-bit ShiftCtrl with n = 4 and n = 3


@pytest.fixture(scope="module")
def sq():
    assert torch.cuda.is_available(), "GPU tests need a device"
    import paper_2105_11010_amd as sq_
    return sq_


def kw(mode):
    n, m, r, p = mode
    return dict(window_bits=n, shift_mask=m, round_nearest=r, pair=p)


def gpu_pack(sq, x, mode, group=1):
    m = sq.mode(*mode)
    xd = torch.from_numpy(x).cuda()
    nbytes = sq.sparq_packed_act_bytes(x.size // x.shape[-1], x.shape[-1], m, group)
    packed = torch.full((nbytes,), 0xAB, dtype=torch.uint8, device="cuda")
    sq.sparq_pack_act(xd, packed, m, group)
    y = torch.full(x.shape, 0xCD, dtype=torch.uint8, device="cuda")
    sq.sparq_unpack_act(packed, y, m, group)
    torch.cuda.synchronize()
    return packed.cpu().numpy(), y.cpu().numpy()


@pytest.mark.parametrize("mode", MODES, ids=str)
def test_every_pair_of_values(sq, oracle, mode):
    a, b = np.meshgrid(np.arange(256), np.arange(256), indexing="ij")
    x = np.stack([a.ravel(), b.ravel()], axis=1).astype(np.uint8).reshape(-1, 64)
    packed, y = gpu_pack(sq, x, mode)
    ref = oracle.pack_act(x, **kw(mode))
    assert np.array_equal(packed.reshape(ref.shape), ref), "records differ from the oracle's"
    assert np.array_equal(y, oracle.trim(x, **kw(mode))), "round trip is not the trim"


@pytest.mark.parametrize("C", [1, 2, 3, 31, 32, 33, 65, 96, 159, 256])
@pytest.mark.parametrize("mode", [(4, S.OPT5, 1, 1), (4, S.OPT3, 0, 1), (4, S.OPT2, 1, 0), (2, S.OPT7_2B, 1, 1)], ids=str)
def test_ragged_channel_counts_and_rows(sq, oracle, C, mode):
    x = S.gen_activations((3, 37, C), 0.5, S.rng_for(7, C))
    packed, y = gpu_pack(sq, x, mode)
    ref = oracle.pack_act(x, **kw(mode))
    assert np.array_equal(packed.reshape(ref.shape), ref)
    assert np.array_equal(y, oracle.unpack_act(ref, x.shape, **kw(mode)))
    assert np.array_equal(y, oracle.trim(x, **kw(mode)))


@pytest.mark.parametrize("group", [2, 4, 8, 16, 32])
@pytest.mark.parametrize("mode", [(4, S.OPT5, 0, 0), (4, S.OPT5, 1, 0), (4, S.OPT3, 1, 0), (4, S.OPT2, 0, 0), (3, S.OPT6_3B, 1, 0),
                                  (2, S.OPT7_2B, 0, 0)], ids=str)
def test_shared_shift_groups(sq, oracle, group, mode):
    x = S.gen_activations((1000, 96), 0.5, S.rng_for(7, 100 + group))
    x[0] = 0
    x[1] = 255
    x[2, ::group] = 255
    packed, y = gpu_pack(sq, x, mode, group)
    ref = oracle.pack_act(x, group, **kw(mode))
    assert np.array_equal(packed.reshape(ref.shape), ref)
    assert np.array_equal(y, oracle.unpack_act(ref, x.shape, group, **kw(mode)))


def test_sizes_and_rejections(sq, oracle):
    for mode in MODES:
        for group in (1, 2, 8, 32):
            want = oracle.packed_record_bytes(group, **kw(mode))
            assert sq.sparq_packed_act_bytes(5, 70, sq.mode(*mode), group) == 5 * 3 * want
    m = sq.mode(4, S.OPT5, 1, 1)
    x = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
    small = torch.zeros(10, dtype=torch.uint8, device="cuda")
    with pytest.raises(sq.SparqError) as e:
        sq.sparq_pack_act(x, small, m)
    assert e.value.status == 3
    with pytest.raises(sq.SparqError):
        sq.sparq_pack_act(x, torch.zeros(4096, dtype=torch.uint8, device="cuda"), sq.mode(8, 1, 0, 0))
    with pytest.raises(sq.SparqError):
        sq.sparq_pack_act(x, torch.zeros(4096, dtype=torch.uint8, device="cuda"), m, 4)       # shared shift needs vSPARQ off
    sq.sparq_pack_act(x[:0], small, m)                                                       # no rows: nothing to do


@pytest.mark.parametrize("layer,group", [
    (S.ConvLayer("p_1x1_256_64", 4, 28, 28, 256, 64, 1, 1, (1, 1), (0, 0), 0.5, S.Mode(4, S.OPT3, 0, 1)), 1),
    (S.ConvLayer("p_3x3_64_96", 2, 17, 17, 64, 96, 3, 3, (1, 1), (1, 1), 0.4, S.Mode(4, S.OPT5, 1, 1)), 1),
    (S.ConvLayer("p_3x3s2_65_48", 2, 19, 19, 65, 48, 3, 3, (2, 2), (1, 1), 0.5, S.Mode(4, S.OPT2, 1, 1)), 1),
    (S.ConvLayer("p_1x1_512_128_g8", 2, 14, 14, 512, 128, 1, 1, (1, 1), (0, 0), 0.5, S.Mode(4, S.OPT5, 1, 0)), 8),
    (S.ConvLayer("p_1x7_160_g4", 2, 17, 17, 160, 160, 1, 7, (1, 1), (0, 3), 0.5, S.Mode(3, S.OPT6_3B, 0, 0)), 4)], ids=lambda v: getattr(v, "name", v))
def test_convolution_on_packed_input(sq, oracle, layer, group):
    """Packed input -> the same int32 accumulators as the oracle's convolution over the values the oracle unpacks."""
    x, w, sc = S.gen_layer(8, layer)
    d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
    m = sq.mode(*layer.mode.astuple())
    dev = torch.device("cuda:0")
    xd, wd, sd = (torch.from_numpy(a).to(dev) for a in (x, w, sc))
    px = torch.empty(sq.sparq_packed_act_bytes(layer.B * layer.H * layer.W, layer.C, m, group), dtype=torch.uint8, device=dev)
    sq.sparq_pack_act(xd, px, m, group)
    pw = torch.empty(sq.sparq_packed_bytes(d), dtype=torch.uint8, device=dev)
    sq.sparq_pack_weights(wd, d, pw)
    ws = torch.empty(sq.sparq_conv_packed_workspace_bytes(d, m), dtype=torch.uint8, device=dev)
    acc = torch.empty((layer.M, layer.N), dtype=torch.int32, device=dev)
    out = torch.empty((layer.M, layer.N), dtype=torch.float32, device=dev)
    sq.sparq_conv_gemm_packed(px, group, pw, d, m, acc=acc, scale=sd, out=out, workspace=ws)
    torch.cuda.synchronize()
    values = oracle.unpack_act(oracle.pack_act(x, group, **layer.mode.kwargs()), x.shape, group, **layer.mode.kwargs())
    if group == 1:
        assert np.array_equal(values, oracle.trim(x, **layer.mode.kwargs()))
    ref_acc, ref_out = oracle.conv_gemm(values, w, layer.stride, layer.pad, scale=sc, **S.PLAIN8.kwargs())
    assert np.array_equal(acc.cpu().numpy(), ref_acc)
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - ref_out) <= 1e-6 * np.abs(ref_out))
    if group == 1:      # and the per-value format gives what the fused convolution gives on the raw input
        acc2 = torch.empty_like(acc)
        wsb = sq.sparq_workspace_bytes(d, m)
        sq.sparq_conv_gemm(xd, pw, d, m, acc=acc2, workspace=torch.empty(wsb, dtype=torch.uint8, device=dev) if wsb else None)
        assert torch.equal(acc, acc2)
