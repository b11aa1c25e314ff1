"""GPU parity of the per-channel reading of Rescaled Magnitude (one factor per channel, Sec. III-B figure captions)
against the CPU oracle.

What is compared how:
  * the two fp64 column sums: the GPU adds the rows in another order than the oracle, so they agree to a few
    units of fp64 rounding, not bit for bit;
  * the fp32 factors: equal, or one fp32 spacing apart where the fp64 quotient falls next to a rounding boundary;
  * the pruned tensor: bit-exact when both sides are given the same factors (the kept set is integer work and the
    product is one fp32 multiplication and one rounding); end to end at most one storage spacing apart;
  * the fused product, which folds the factors into the filter rows instead of the gradient: the stated tolerance
    of the backward-data product (1e-2 bf16, 1e-5 fp32, relative to sum |dO||W|).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_00774_amd as sdgp
from paper_2202_00774_amd import workloads as wl
from util import rel_error, to_gpu, to_host

pytestmark = pytest.mark.gpu

DTYPES = [oracle.BF16, oracle.F32]
NM = [(2, 4), (1, 4), (2, 8), (4, 8), (2, 16), (4, 16), (2, 32), (16, 32), (3, 5), (2, 6), (4, 4)]
# rows x groups: one group per row, several workgroups down the rows, a slot count that is no power of two, and more
# slots than a workgroup is wide (two workgroups side by side, the second one partly idle)
SHAPES = [(37, 1), (1000, 3), (4099, 16), (300, 47), (70, 600)]


def ulp_distance_f32(a, b):
    ia, ib = a.view(np.int32).astype(np.int64), b.view(np.int32).astype(np.int64)
    return np.abs(ia - ib)


def check_scales(dO_host, n, m):
    C = dO_host.shape[-1]
    _, ref_scale, ref_total, ref_kept = oracle.prune_channel_rescaled(dO_host.reshape(-1, C), n, m)
    d = to_gpu(dO_host)
    before = d.clone()
    scale, sums = sdgp.sdgp_channel_scales(d, n, m, sums=True)
    torch.cuda.synchronize()
    assert torch.equal(d.view(torch.uint8), before.view(torch.uint8))
    sums = sums.cpu().numpy()
    scale = scale.cpu().numpy()
    assert np.all(np.abs(sums[0] - ref_total) <= 1e-13 * ref_total)
    assert np.all(np.abs(sums[1] - ref_kept) <= 1e-13 * ref_kept)
    assert np.array_equal(sums[1] == 0, ref_kept == 0)
    dist = ulp_distance_f32(scale, ref_scale)
    assert dist.max(initial=0) <= 1
    assert np.count_nonzero(dist) <= max(1, C // 1000)
    # the same bits from call to call (fixed order of the partial sums)
    again = sdgp.sdgp_channel_scales(d, n, m)
    assert np.array_equal(again.cpu().numpy().view(np.int32), scale.view(np.int32))
    return d, scale, ref_scale


def check_prune(dO_host, n, m):
    C = dO_host.shape[-1]
    ref_pruned, ref_scale, _, _ = oracle.prune_channel_rescaled(dO_host.reshape(-1, C), n, m)
    ref_pruned = ref_pruned.reshape(dO_host.shape)
    d, scale, _ = check_scales(dO_host, n, m)
    # same factors in: same bits out
    got = sdgp.sdgp_prune_channel_rescaled(d, n, m, scale=torch.from_numpy(ref_scale).cuda())
    assert np.array_equal(to_host(got).view(np.uint8), ref_pruned.view(np.uint8))
    # end to end: factors from the GPU
    got = to_host(sdgp.sdgp_prune_channel_rescaled(d, n, m))
    if got.dtype == np.uint16:
        a, b = got.astype(np.int64), ref_pruned.astype(np.int64)
    else:
        a, b = got.view(np.int32).astype(np.int64), ref_pruned.view(np.int32).astype(np.int64)
    assert np.abs(a - b).max(initial=0) <= 1
    assert np.count_nonzero(a != b) <= max(1, got.size // 1000)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n,m", NM)
def test_scales_and_pruned_tensor_match_oracle(dtype, n, m):
    for rows, groups in SHAPES:
        dO = wl.laplace_with_zeros((rows, groups * m), 1e-3, 0.3, seed=7 * m + n + rows, dtype=dtype)
        check_prune(dO, n, m)


@pytest.mark.parametrize("dtype", DTYPES)
def test_tiny_ragged_and_degenerate(dtype):
    for rows, C, n, m in ((1, 4, 2, 4), (1, 8, 2, 4), (2, 12, 2, 4), (3, 20, 2, 4), (1, 16, 2, 16), (65, 8, 2, 8),
                          (1, 32, 4, 32), (63, 36, 2, 4), (129, 24, 3, 8)):
        dO = wl.laplace_with_zeros((rows, C), 1.0, 0.4, seed=rows * 100 + C, dtype=dtype)
        check_prune(dO, n, m)
    # a channel that is zero in every row, and one that is never kept: factor 1, output +0
    dO = wl.laplace_with_zeros((500, 16), 1.0, 0.0, seed=5, dtype=oracle.F32)
    dO = np.abs(dO) + 1.0
    dO[:, 3] = 0.0
    dO[:, 6] = 1e-3
    dO = wl.to_storage(dO, dtype)
    d, scale, ref_scale = check_scales(dO, 2, 4)
    assert scale[3] == 1.0 and scale[6] == 1.0 and ref_scale[3] == 1.0 and ref_scale[6] == 1.0
    check_prune(dO, 2, 4)
    # all zeros, with signs
    z = np.zeros((40, 32), np.float32)
    z[::2] = -0.0
    check_prune(wl.to_storage(z, dtype), 2, 4)


def test_empty_tensors():
    for shape in ((0, 16), (4, 0)):
        d = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
        scale = sdgp.sdgp_channel_scales(d, 2, 4)
        assert scale.shape == (shape[1],)
        if shape[1]:
            assert torch.all(scale == 1.0)
        assert sdgp.sdgp_prune_channel_rescaled(d, 2, 4).shape == shape


@pytest.mark.parametrize("dtype", DTYPES)
def test_unaligned_pointers_take_the_scalar_path(dtype):
    rows, C, n, m = 200, 64, 2, 4
    dO = wl.laplace_with_zeros((rows, C), 1e-3, 0.3, seed=77, dtype=dtype)
    ref_pruned, ref_scale, _, _ = oracle.prune_channel_rescaled(dO, n, m)
    flat = to_gpu(np.concatenate([dO.reshape(-1)[:1], dO.reshape(-1)]))
    d = flat[1:].view(rows, C)          # element size away from 16-byte alignment
    assert d.data_ptr() % 16 != 0
    scale = sdgp.sdgp_channel_scales(d, n, m)
    assert ulp_distance_f32(scale.cpu().numpy(), ref_scale).max() <= 1
    got = sdgp.sdgp_prune_channel_rescaled(d, n, m, scale=torch.from_numpy(ref_scale).cuda())
    assert np.array_equal(to_host(got).view(np.uint8), ref_pruned.view(np.uint8))


@pytest.mark.parametrize("dtype", DTYPES)
def test_scale_filter_is_one_fp32_product_and_one_rounding(dtype):
    rng = np.random.default_rng(4)
    W = wl.normal((48, 3, 3, 24), 0.05, seed=9, dtype=dtype)
    s = (1.0 + rng.random(48)).astype(np.float32)
    wf = wl.bf16_bits_to_f32(W) if dtype == oracle.BF16 else W
    want = wl.to_storage(wf * s[:, None, None, None], dtype)      # numpy fp32 product, then the storage rounding
    Wg, sg = to_gpu(W), torch.from_numpy(s).cuda()
    got = sdgp.sdgp_scale_filter(Wg, sg)
    assert np.array_equal(to_host(got).view(np.uint8), want.view(np.uint8))
    # in place
    sdgp.sdgp_scale_filter(Wg, sg, out=Wg)
    assert np.array_equal(to_host(Wg).view(np.uint8), want.view(np.uint8))


LAYERS = [
    # name, B, H, W, C_in, C_out, R, S, stride, pad
    ("c3x3", 4, 16, 16, 64, 128, 3, 3, 1, 1),
    ("c3x3_wide", 2, 8, 8, 256, 256, 3, 3, 1, 1),
    ("pw", 3, 14, 14, 128, 64, 1, 1, 1, 0),
    ("pw_s2", 2, 14, 14, 64, 128, 1, 1, 2, 0),
    ("c3x3_s2", 2, 16, 16, 64, 64, 3, 3, 2, 1),
    ("stem", 2, 12, 12, 3, 64, 3, 3, 1, 1),
    ("odd", 2, 7, 9, 24, 40, 3, 3, 1, 1),
    ("stem5x5", 2, 20, 20, 2, 64, 5, 5, 1, 2),      # first-layer kernel, filter gathered inside the kernel (no filter image here)
    # a wide first-layer filter (five column tiles of (tap, channel) pairs): sdgp_conv_bwd_data would build a transposed
    # image of it in its workspace; this entry point hands the first-layer kernel no workspace, so the kernel gathers
    # the filter itself
    ("stem7x7s2", 2, 30, 30, 3, 64, 7, 7, 2, 3),
]


def check_conv(layer, n, m, dtype, seed):
    name, B, H, Wd, C_in, C_out, R, S, stride, pad = layer
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    dO = wl.laplace_with_zeros((B, P, Q, C_out), 1e-3, 0.3, seed=seed, dtype=dtype)
    W = wl.normal((C_out, R, S, C_in), (2.0 / (R * S * C_in)) ** 0.5, seed=seed + 1, dtype=dtype)
    pruned, _, _, _ = oracle.prune_channel_rescaled(dO.reshape(-1, C_out), n, m)
    ref, absum = oracle.conv_bwd_data(pruned.reshape(dO.shape), W, H, Wd, stride, pad)
    got = sdgp.sdgp_conv_bwd_data_channel_rescaled(to_gpu(dO), to_gpu(W), H, Wd, stride, pad, n, m)
    got = wl.to_f64(to_host(got))
    tol = 1e-2 if dtype == oracle.BF16 else 1e-5
    err = rel_error(got, ref, absum)
    assert err <= tol, (name, n, m, err)
    # pixels no tap reaches (stride > 1) are zero on both sides
    assert np.all(got[absum == 0] == 0)
    return err


@pytest.mark.parametrize("layer", LAYERS, ids=[l[0] for l in LAYERS])
@pytest.mark.parametrize("n,m", [(2, 4), (2, 8), (2, 16), (4, 8)])
def test_fused_conv_matches_oracle_bf16(layer, n, m):
    if layer[5] % m:
        pytest.skip("C_out is not a multiple of m")
    check_conv(layer, n, m, oracle.BF16, seed=31 * m + n)


@pytest.mark.parametrize("layer", [LAYERS[0], LAYERS[2], LAYERS[6]], ids=lambda l: l[0])
def test_fused_conv_matches_oracle_fp32(layer):
    check_conv(layer, 2, 4, oracle.F32, seed=3)


@pytest.mark.parametrize("dtype", DTYPES)
def test_fused_linear_matches_oracle(dtype):
    rows, C_out, C_in, n, m = 300, 128, 96, 2, 4
    dO = wl.normal((rows, C_out), 1.0, seed=1, dtype=dtype)
    W = wl.normal((C_out, C_in), (1.0 / C_out) ** 0.5, seed=2, dtype=dtype)
    pruned, _, _, _ = oracle.prune_channel_rescaled(dO, n, m)
    ref, absum = oracle.linear_bwd_data(pruned, W)
    got = wl.to_f64(to_host(sdgp.sdgp_linear_bwd_data_channel_rescaled(to_gpu(dO), to_gpu(W), n, m)))
    assert rel_error(got, ref, absum) <= (1e-2 if dtype == oracle.BF16 else 1e-5)


def test_no_output_channels_gives_zeros():
    """C_out = 0: an empty sum for every element of dL/dD."""
    B, H, Wd, C_in = 2, 6, 5, 8
    dO = torch.empty((B, H, Wd, 0), dtype=torch.bfloat16, device="cuda")
    W = torch.empty((0, 3, 3, C_in), dtype=torch.bfloat16, device="cuda")
    out = torch.full((B, H, Wd, C_in), 7.0, dtype=torch.bfloat16, device="cuda")
    sdgp.sdgp_conv_bwd_data_channel_rescaled(dO, W, H, Wd, 1, 1, 2, 4, out=out)
    assert torch.all(out == 0)
    out.fill_(7.0)
    sdgp.sdgp_conv_bwd_data(dO, W, H, Wd, 1, 1, 2, 4, sdgp.GREEDY, out=out)
    assert torch.all(out == 0)


def test_fused_equals_its_three_steps():
    # the one-call entry point is channel scales -> rescaled filter -> fused Magnitude product, bit for bit
    B, H, Wd, C_in, C_out = 4, 16, 16, 64, 128
    dO = to_gpu(wl.laplace_with_zeros((B, H, Wd, C_out), 1e-3, 0.3, seed=8, dtype=oracle.BF16))
    W = to_gpu(wl.normal((C_out, 3, 3, C_in), 0.06, seed=9, dtype=oracle.BF16))
    one = sdgp.sdgp_conv_bwd_data_channel_rescaled(dO, W, H, Wd, 1, 1, 2, 4)
    scale = sdgp.sdgp_channel_scales(dO, 2, 4)
    three = sdgp.sdgp_conv_bwd_data(dO, sdgp.sdgp_scale_filter(W, scale), H, Wd, 1, 1, 2, 4, sdgp.GREEDY)
    assert torch.equal(one.view(torch.int16), three.view(torch.int16))


def test_resnet9_layer_at_full_size():
    """64 -> 128 channels at 32x32, batch 512 (the largest layer of the ResNet-9 sweep): factors over 524288 rows,
    the pruned tensor bit-exact given the oracle's factors, the fused product at sampled pixels."""
    layer = [l for l in wl.resnet9_layers(512) if l.C_in == 64 and l.C_out == 128][0]
    dO, W = wl.layer_inputs(layer, 1e-3, 0.3, seed=2001)
    C = layer.C_out
    ref_pruned, ref_scale, ref_total, ref_kept = oracle.prune_channel_rescaled(dO.reshape(-1, C), 2, 4)
    d = to_gpu(dO)
    scale, sums = sdgp.sdgp_channel_scales(d, 2, 4, sums=True)
    sums = sums.cpu().numpy()
    assert np.all(np.abs(sums[0] - ref_total) <= 1e-12 * ref_total)
    assert np.all(np.abs(sums[1] - ref_kept) <= 1e-12 * ref_kept)
    assert ulp_distance_f32(scale.cpu().numpy(), ref_scale).max() <= 1
    got = sdgp.sdgp_prune_channel_rescaled(d, 2, 4, scale=torch.from_numpy(ref_scale).cuda())
    assert torch.equal(got.view(torch.int16).cpu(), torch.from_numpy(ref_pruned.view(np.int16)).view(got.shape))
    del got
    rng = np.random.default_rng(0)
    H, Wd = layer.H, layer.Wd
    corners = [0, Wd - 1, (H - 1) * Wd, H * Wd - 1, (layer.B - 1) * H * Wd, layer.B * H * Wd - 1]
    pixels = np.unique(np.concatenate([np.array(corners), rng.integers(0, layer.B * H * Wd, 2048)]))
    ref, absum = oracle.conv_bwd_data(ref_pruned.reshape(dO.shape), W, H, Wd, layer.stride, layer.pad, pixels=pixels)
    out = sdgp.sdgp_conv_bwd_data_channel_rescaled(d, to_gpu(W), H, Wd, layer.stride, layer.pad, 2, 4)
    idx = torch.from_numpy(pixels).cuda()
    sample = wl.to_f64(to_host(out.view(-1, layer.C_in)[idx]))
    assert rel_error(sample, ref, absum) <= 1e-2


def test_bench_tensor_at_full_size():
    """The tensor bench.py times the sweep on ([3211264, 64] bf16, 411 MB, 2:4): sums, factors and the pruned tensor."""
    rows, C = 256 * 112 * 112, 64
    dO = wl.laplace_with_zeros((rows, C), 1e-3, 0.3, seed=9000, dtype=oracle.BF16)
    ref_pruned, ref_scale, ref_total, ref_kept = oracle.prune_channel_rescaled(dO, 2, 4)
    d = to_gpu(dO)
    scale, sums = sdgp.sdgp_channel_scales(d, 2, 4, sums=True)
    sums = sums.cpu().numpy()
    assert np.all(np.abs(sums[0] - ref_total) <= 1e-12 * ref_total)
    assert np.all(np.abs(sums[1] - ref_kept) <= 1e-12 * ref_kept)
    assert ulp_distance_f32(scale.cpu().numpy(), ref_scale).max() <= 1
    got = sdgp.sdgp_prune_channel_rescaled(d, 2, 4, scale=torch.from_numpy(ref_scale).cuda())
    assert torch.equal(got.view(torch.int16).cpu(), torch.from_numpy(ref_pruned.view(np.int16)).view(got.shape))
