"""GPU parity of the forward convolution and the weight gradient (Sec. II-A, Fig. 1; Sec. III-A) against the oracle.

Tolerances, relative to the sum of |a||b| over the terms of an output element (the oracle returns it):
  forward        1e-2: bf16 inputs, fp32 accumulation, one bf16 rounding of the result (2^-9 of the value) -- the
                 bar of the backward-data product, whose kernels compute it;
  weight gradient 1e-3: fp32 accumulation of up to 5e5 products and an fp32 result: the rounding of a sum of N terms
                 grows like sqrt(N) * 2^-24 (4e-5 at the largest N here); nothing is rounded to bf16.
  fp32 layers    1e-5 (forward), 1e-4 (weight gradient).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_00774_amd as sdgp
from paper_2202_00774_amd import workloads as wl
from util import to_gpu, to_host

pytestmark = pytest.mark.gpu


def inputs(L, seed, dtype=wl.BF16):
    D = wl.normal(L.dD_shape, 1.0, seed, dtype)
    W = wl.normal(L.W_shape, float(np.sqrt(2.0 / (L.R * L.S * L.C_in))), seed + 1, dtype)
    G = wl.laplace_with_zeros(L.dO_shape, 1e-3, 0.3, seed + 2, dtype)
    return D, W, G


def check_fwd(L, D, W, tol, pixels=None):
    ref, ab = oracle.conv_fwd(D, W, L.stride, L.pad, pixels=pixels)
    out = sdgp.sdgp_conv_fwd(to_gpu(D), to_gpu(W), L.stride, L.pad)
    torch.cuda.synchronize()
    assert tuple(out.shape) == L.dO_shape
    got = to_host(out)
    if pixels is not None:
        got = got.reshape(-1, L.C_out)[pixels]
    got = wl.to_f64(got)
    err = np.abs(got - ref) / (ab + 1e-300)
    assert np.all(got[ab == 0] == 0)
    assert err[ab > 0].max() <= tol, (L.name, err.max())


def check_wgrad(L, D, G, tol, entries=None):
    ref, ab = oracle.conv_bwd_weight(D, G, L.R, L.S, L.stride, L.pad, entries=entries)
    out = sdgp.sdgp_conv_bwd_weight(to_gpu(D), to_gpu(G), L.R, L.S, L.stride, L.pad)
    again = sdgp.sdgp_conv_bwd_weight(to_gpu(D), to_gpu(G), L.R, L.S, L.stride, L.pad)
    torch.cuda.synchronize()
    assert tuple(out.shape) == L.W_shape and out.dtype == torch.float32
    assert torch.equal(out, again)                       # partial sums are added in a fixed order
    got = out.cpu().numpy().astype(np.float64)
    if entries is not None:
        got = got.reshape(-1)[entries]
    err = np.abs(got - ref) / (ab + 1e-300)
    assert np.all(got[ab == 0] == 0)
    assert err[ab > 0].max() <= tol, (L.name, err.max())


# matrix-core weight-gradient kernel: 3x3 stride 1, channel counts multiples of 64; several tiles per image, ragged
# last tile, rows that are not a multiple of four pixels, pads 0..2, blocks of 64 and of 128 output channels
MFMA_LAYERS = [
    wl.ConvLayer("w16_64x128", 6, 16, 16, 64, 128, 3, 3, 1, 1),
    wl.ConvLayer("w32_64x64", 3, 32, 32, 64, 64, 3, 3, 1, 1),
    wl.ConvLayer("w8_128x256", 5, 8, 8, 128, 256, 3, 3, 1, 1),
    wl.ConvLayer("w4_128x128", 9, 4, 4, 128, 128, 3, 3, 1, 1),
    wl.ConvLayer("w14_64x64", 4, 14, 14, 64, 64, 3, 3, 1, 1),
    wl.ConvLayer("w20_ragged_64x192", 2, 20, 20, 64, 192, 3, 3, 1, 1),
    wl.ConvLayer("w12_pad0_64x128", 3, 12, 13, 64, 128, 3, 3, 1, 0),
    wl.ConvLayer("w10_pad2_128x64", 2, 10, 9, 128, 64, 3, 3, 1, 2),
    wl.ConvLayer("w56_64x64", 1, 56, 56, 64, 64, 3, 3, 1, 1),
]
# plain kernels: stride 2, 1x1, a 7x7 first layer, channel counts the matrix-core kernels do not take
PLAIN_LAYERS = [
    wl.ConvLayer("s2_3x3", 2, 15, 14, 32, 48, 3, 3, 2, 1),
    wl.ConvLayer("pw_1x1", 2, 9, 9, 64, 128, 1, 1, 1, 0),
    wl.ConvLayer("pw_1x1_s2", 2, 9, 10, 24, 40, 1, 1, 2, 0),
    wl.ConvLayer("stem_7x7", 2, 30, 30, 3, 64, 7, 7, 2, 3),
    wl.ConvLayer("first_3x3", 3, 16, 16, 3, 64, 3, 3, 1, 1),
    wl.ConvLayer("first_wide_rows", 2, 12, 70, 3, 128, 3, 3, 1, 1),      # two segments per row, the second ragged
    wl.ConvLayer("first_many", 300, 9, 9, 4, 64, 3, 3, 1, 1),            # more segments than workgroups
    wl.ConvLayer("stem_7x7_wide", 1, 40, 150, 3, 64, 7, 7, 2, 3),
    wl.ConvLayer("odd_5x5", 2, 11, 12, 20, 36, 5, 5, 1, 2),
    wl.ConvLayer("rect_2x3", 2, 8, 9, 16, 32, 2, 3, 1, 1),
]


@pytest.mark.parametrize("L", MFMA_LAYERS + PLAIN_LAYERS, ids=lambda L: L.name)
def test_weight_gradient_matches_oracle(L):
    D, _, G = inputs(L, 100 + L.C_out + L.H)
    check_wgrad(L, D, G, 1e-3)


@pytest.mark.parametrize("L", MFMA_LAYERS + PLAIN_LAYERS, ids=lambda L: L.name)
def test_forward_matches_oracle(L):
    D, W, _ = inputs(L, 200 + L.C_out + L.H)
    check_fwd(L, D, W, 1e-2)


@pytest.mark.parametrize("L", [MFMA_LAYERS[0], PLAIN_LAYERS[0], PLAIN_LAYERS[1]], ids=lambda L: L.name)
def test_fp32_layers(L):
    D, W, G = inputs(L, 300, wl.F32)
    check_fwd(L, D, W, 1e-5)
    check_wgrad(L, D, G, 1e-4)


def test_weight_gradient_reads_every_gradient_element():
    """The gradient is taken unpruned: a tensor whose only nonzero is the smallest magnitude of its group still counts."""
    L = wl.ConvLayer("w8_64x64", 1, 8, 8, 64, 64, 3, 3, 1, 1)
    D = wl.normal(L.dD_shape, 1.0, 1, wl.BF16)
    G = np.zeros(L.dO_shape, np.uint16)
    G[0, 3, 4, :] = wl.f32_to_bf16_bits(np.linspace(1, 64, 64).astype(np.float32))   # every channel of one pixel
    check_wgrad(L, D, G, 1e-3)
    out = sdgp.sdgp_conv_bwd_weight(to_gpu(D), to_gpu(G), 3, 3, 1, 1).cpu().numpy()
    assert np.all(out[:, 1, 1, :] != 0)


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4, 5])
def test_resnet9_batch512_sampled(i):
    """The launches bench.py times: forward at sampled output pixels, weight gradient at sampled filter elements."""
    L = wl.resnet9_layers(512)[i]
    D, W, G = inputs(L, 400 + i)
    rng = np.random.default_rng(i)
    npix = L.B * L.P * L.Q
    pixels = np.unique(np.concatenate([[0, L.Q - 1, npix - 1], rng.integers(0, npix, 300)]))
    check_fwd(L, D, W, 1e-2, pixels=pixels)
    nW = int(np.prod(L.W_shape))
    entries = np.unique(np.concatenate([[0, nW - 1, L.C_in * 4], rng.integers(0, nW, 160)]))
    check_wgrad(L, D, G, 1e-3, entries=entries)


def test_empty_and_errors():
    x = torch.zeros((0, 8, 8, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((64, 3, 3, 64), dtype=torch.bfloat16, device="cuda")
    assert sdgp.sdgp_conv_fwd(x, w, 1, 1).shape == (0, 8, 8, 64)
    g = torch.zeros((0, 8, 8, 64), dtype=torch.bfloat16, device="cuda")
    assert not sdgp.sdgp_conv_bwd_weight(x, g, 3, 3, 1, 1).any()          # an empty sum per filter element
    with pytest.raises(sdgp.SdgpError):
        sdgp.sdgp_conv_fwd(torch.zeros((1, 2, 2, 8), dtype=torch.bfloat16, device="cuda"),
                           torch.zeros((8, 3, 3, 8), dtype=torch.bfloat16, device="cuda"), 1, 3)   # pad >= R
