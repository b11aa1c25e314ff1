"""Pins for the CPU oracle's grouped backward-data product (the RegNetX layers of Sec. IV use group convolutions).

Expectations come from the input gradient of torch's fp64 grouped conv2d (the library routine the sum reduces to),
from the ungrouped oracle on a block-diagonal filter (a grouped convolution is a convolution whose filter is zero
outside the diagonal blocks), from the groups == 1 case, from a one-hot example, and from the depthwise case
written out by hand.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_00774_amd import workloads as wl

GEOMS = [
    # B, H, Wd, C_in, C_out, R, S, stride, pad, groups
    (2, 7, 6, 8, 12, 3, 3, 1, 1, 4),
    (1, 9, 9, 6, 6, 3, 3, 2, 1, 3),
    (2, 5, 8, 16, 8, 1, 1, 1, 0, 8),
    (1, 8, 8, 4, 4, 3, 3, 1, 1, 4),      # depthwise
    (2, 6, 6, 6, 9, 2, 3, 1, 1, 3),
    (1, 11, 10, 4, 8, 5, 5, 2, 2, 2),
]


def torch_grouped_input_grad(dO, W, H, Wd, stride, pad, groups):
    B, P, Q, C_out = dO.shape
    _, R, S, cig = W.shape
    x = torch.zeros((B, cig * groups, H, Wd), dtype=torch.float64, requires_grad=True)
    w = torch.from_numpy(W.transpose(0, 3, 1, 2).copy())
    y = torch.nn.functional.conv2d(x, w, stride=stride, padding=pad, groups=groups)
    assert tuple(y.shape) == (B, C_out, P, Q)
    y.backward(torch.from_numpy(dO.transpose(0, 3, 1, 2).copy()))
    return x.grad.numpy().transpose(0, 2, 3, 1)


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_grouped_matches_torch_input_gradient(geom, dtype):
    B, H, Wd, C_in, C_out, R, S, stride, pad, groups = geom
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    dO = wl.normal((B, P, Q, C_out), 1.0, 3, dtype)
    W = wl.normal((C_out, R, S, C_in // groups), 0.5, 4, dtype)
    dD, ab = oracle.conv_bwd_data_grouped(dO, W, H, Wd, stride, pad, groups)
    want = torch_grouped_input_grad(wl.to_f64(dO), wl.to_f64(W), H, Wd, stride, pad, groups)
    assert np.allclose(dD, want, rtol=1e-12, atol=1e-12)
    want_ab = torch_grouped_input_grad(np.abs(wl.to_f64(dO)), np.abs(wl.to_f64(W)), H, Wd, stride, pad, groups)
    assert np.allclose(ab, want_ab, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("geom", GEOMS)
def test_grouped_is_a_block_diagonal_filter(geom):
    B, H, Wd, C_in, C_out, R, S, stride, pad, groups = geom
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    dO = wl.normal((B, P, Q, C_out), 1.0, 5, oracle.F32)
    W = wl.normal((C_out, R, S, C_in // groups), 0.5, 6, oracle.F32)
    cig, cog = C_in // groups, C_out // groups
    full = np.zeros((C_out, R, S, C_in), np.float32)
    for g in range(groups):
        full[g * cog:(g + 1) * cog, :, :, g * cig:(g + 1) * cig] = W[g * cog:(g + 1) * cog]
    a, _ = oracle.conv_bwd_data_grouped(dO, W, H, Wd, stride, pad, groups)
    b, _ = oracle.conv_bwd_data(dO, full, H, Wd, stride, pad)
    assert np.array_equal(a, b)           # the same terms in the same order, plus exact zeros


def test_one_group_is_the_plain_product():
    dO = wl.normal((2, 5, 5, 8), 1.0, 7, oracle.BF16)
    W = wl.normal((8, 3, 3, 6), 0.5, 8, oracle.BF16)
    a, aa = oracle.conv_bwd_data_grouped(dO, W, 5, 5, 1, 1, 1)
    b, bb = oracle.conv_bwd_data(dO, W, 5, 5, 1, 1)
    assert np.array_equal(a, b) and np.array_equal(aa, bb)


def test_one_hot_gradient_reaches_only_its_group():
    """dO = 1 at output channel 5 (group 1 of 3, with 2 input and 3 output channels per group): only input channels
    2 and 3 receive anything, and they receive the filter taps of output channel 5."""
    dO = np.zeros((1, 4, 4, 9), np.float32)
    dO[0, 1, 2, 5] = 1.0
    W = wl.normal((9, 3, 3, 2), 1.0, 9, oracle.F32)
    dD, _ = oracle.conv_bwd_data_grouped(dO, W, 4, 4, 1, 1, 3)
    assert not dD[..., [0, 1, 4, 5]].any()
    for r in range(3):
        for s in range(3):
            h, w = 1 + r - 1, 2 + s - 1       # output pixel (1,2) read input pixel (1 + r - pad, 2 + s - pad) at tap (r,s)
            if 0 <= h < 4 and 0 <= w < 4:
                assert dD[0, h, w, 2] == W[5, r, s, 0] and dD[0, h, w, 3] == W[5, r, s, 1]


def test_depthwise_by_hand():
    """One channel per group, 1x3 filter, stride 1, no padding, one row of six input pixels and four output pixels:
    output q read inputs q .. q+2, so dD[w] = sum_s dO[w - s] * W[s] over the s with 0 <= w - s < 4."""
    x = [1.0, 2.0, 4.0, 8.0]
    dO = np.zeros((1, 1, 4, 2), np.float32)
    dO[0, 0, :, 0] = x
    dO[0, 0, :, 1] = [-v for v in x]
    taps = ([1.0, 10.0, 100.0], [3.0, 5.0, 7.0])
    W = np.array(taps, np.float32).reshape(2, 1, 3, 1)
    got, _ = oracle.conv_bwd_data_grouped(dO, W, 1, 6, 1, 0, 2)
    want0 = [sum(x[w - s] * taps[0][s] for s in range(3) if 0 <= w - s < 4) for w in range(6)]
    want1 = [-sum(x[w - s] * taps[1][s] for s in range(3) if 0 <= w - s < 4) for w in range(6)]
    assert want0 == [1.0, 12.0, 124.0, 248.0, 480.0, 800.0]
    assert got[0, 0, :, 0].tolist() == want0 and got[0, 0, :, 1].tolist() == want1


def test_sampled_pixels_equal_the_full_result():
    B, H, Wd, C_in, C_out, R, S, stride, pad, groups = GEOMS[0]
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    dO = wl.normal((B, P, Q, C_out), 1.0, 10, oracle.BF16)
    W = wl.normal((C_out, R, S, C_in // groups), 0.5, 11, oracle.BF16)
    full, fab = oracle.conv_bwd_data_grouped(dO, W, H, Wd, stride, pad, groups)
    pix = np.array([0, 5, 17, B * H * Wd - 1])
    part, pab = oracle.conv_bwd_data_grouped(dO, W, H, Wd, stride, pad, groups, pixels=pix)
    assert np.array_equal(part, full.reshape(-1, C_in)[pix]) and np.array_equal(pab, fab.reshape(-1, C_in)[pix])


def test_bad_arguments_are_rejected():
    dO = np.zeros((1, 4, 4, 6), np.float32)
    with pytest.raises(ValueError):
        oracle.conv_bwd_data_grouped(dO, np.zeros((6, 3, 3, 2), np.float32), 4, 4, 1, 1, 4)    # 6 % 4 != 0
