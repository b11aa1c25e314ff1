"""Pins for the oracle's forward convolution and weight gradient (Sec. II-A, Fig. 1; Sec. III-A).

Expectations come from hand-worked cases, from torch's fp64 ``conv2d`` and the weight gradient autograd derives from
it (the library routines these sums are), from an explicit loop over an im2col matrix written here, and from the
adjoint identities that tie the three products of a layer together:
    <conv_fwd(D, W), G> = <D, conv_bwd_data(G, W)> = <W, conv_bwd_weight(D, G)>.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_00774_amd import workloads as wl

GEOMS = [  # B, H, Wd, C_in, C_out, R, S, stride, pad
    (2, 6, 7, 3, 4, 3, 3, 1, 1),
    (2, 8, 8, 4, 6, 3, 3, 2, 1),
    (1, 9, 7, 2, 3, 5, 5, 2, 2),
    (3, 5, 5, 5, 2, 1, 1, 1, 0),
    (2, 7, 6, 3, 5, 1, 1, 2, 0),
    (1, 11, 11, 3, 4, 7, 7, 2, 3),
    (2, 6, 6, 2, 3, 3, 3, 3, 0),
    (2, 4, 5, 3, 2, 2, 3, 1, 1),
]


def tensors(g, dtype, seed=0):
    B, H, Wd, C_in, C_out, R, S, stride, pad = g
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    D = wl.normal((B, H, Wd, C_in), 1.0, 10 + seed, dtype)
    W = wl.normal((C_out, R, S, C_in), 0.5, 20 + seed, dtype)
    G = wl.normal((B, P, Q, C_out), 1.0, 30 + seed, dtype)
    return D, W, G


def as_torch(a):
    return torch.from_numpy(wl.to_f64(a))


def test_hand_worked_forward_and_weight_gradient():
    """One image of 1 x 3 pixels, one channel in and out, filter [1, 2, 4] along the width, pad 1:
    O = [2a+4b, a+2b+4c, b+2c]; with G = [g0, g1, g2]: dW = [g1 a + g2 b, g0 a + g1 b + g2 c, g0 b + g1 c]."""
    a, b, c = 3.0, 5.0, 7.0
    D = np.array([a, b, c], np.float32).reshape(1, 1, 3, 1)
    W = np.array([1, 2, 4], np.float32).reshape(1, 1, 3, 1)
    Dp = np.zeros((1, 3, 3, 1), np.float32)          # the same row between two zero rows, 3 x 3 filter with one live row
    Dp[0, 1, :, 0] = [a, b, c]
    W3 = np.zeros((1, 3, 3, 1), np.float32)
    W3[0, 1, :, 0] = [1, 2, 4]
    O, ab = oracle.conv_fwd(Dp, W3, 1, 1)
    assert O[0, 1, :, 0].tolist() == [2 * a + 4 * b, a + 2 * b + 4 * c, b + 2 * c]
    assert ab[0, 1, :, 0].tolist() == [2 * a + 4 * b, a + 2 * b + 4 * c, b + 2 * c]
    g0, g1, g2 = 1.0, -2.0, 0.5
    G = np.zeros((1, 3, 3, 1), np.float32)
    G[0, 1, :, 0] = [g0, g1, g2]
    dW, ab = oracle.conv_bwd_weight(Dp, G, 3, 3, 1, 1)
    assert dW[0, 1, :, 0].tolist() == [g1 * a + g2 * b, g0 * a + g1 * b + g2 * c, g0 * b + g1 * c]
    assert ab[0, 1, :, 0].tolist() == [2 * a + 0.5 * b, a + 2 * b + 0.5 * c, b + 2 * c]
    # the live gradient row also meets the zero rows of D through the other filter rows: those sums are empty
    assert dW[0, 0, :, 0].tolist() == [0, 0, 0] and dW[0, 2, :, 0].tolist() == [0, 0, 0]


def test_pointwise_layer_is_a_matrix_product():
    """1 x 1, stride 1: O = D W^T per pixel and dW = G^T D (Fig. 1 right)."""
    D, W, G = tensors((2, 4, 5, 6, 3, 1, 1, 1, 0), oracle.F32)
    O, _ = oracle.conv_fwd(D, W, 1, 0)
    d, w, g = D.reshape(-1, 6).astype(np.float64), W.reshape(3, 6).astype(np.float64), G.reshape(-1, 3).astype(np.float64)
    assert np.allclose(O.reshape(-1, 3), d @ w.T, rtol=1e-13, atol=1e-13)
    dW, ab = oracle.conv_bwd_weight(D, G, 1, 1, 1, 0)
    assert np.allclose(dW.reshape(3, 6), g.T @ d, rtol=1e-13, atol=1e-13)
    assert np.allclose(ab.reshape(3, 6), np.abs(g).T @ np.abs(d), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
@pytest.mark.parametrize("g", GEOMS)
def test_forward_and_weight_gradient_match_the_library_in_fp64(g, dtype):
    B, H, Wd, C_in, C_out, R, S, stride, pad = g
    D, W, G = tensors(g, dtype)
    x = as_torch(D).permute(0, 3, 1, 2).clone().requires_grad_(True)
    w = as_torch(W).permute(0, 3, 1, 2).clone().requires_grad_(True)
    y = torch.nn.functional.conv2d(x, w, None, stride, pad)
    O, ab = oracle.conv_fwd(D, W, stride, pad)
    assert np.allclose(O, y.detach().permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    yabs = torch.nn.functional.conv2d(x.detach().abs(), w.detach().abs(), None, stride, pad)
    assert np.allclose(ab, yabs.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    y.backward(as_torch(G).permute(0, 3, 1, 2))
    dW, _ = oracle.conv_bwd_weight(D, G, R, S, stride, pad)
    assert np.allclose(dW, w.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("g", GEOMS[:5])
def test_im2col_products(g):
    """Sec. II-A: with the patches of D as rows of a matrix, forward is patches @ filter^T and dW is G^T @ patches."""
    B, H, Wd, C_in, C_out, R, S, stride, pad = g
    D, W, G = tensors(g, oracle.F32, seed=3)
    P, Q = G.shape[1:3]
    cols = np.zeros((B * P * Q, R * S * C_in))
    for b in range(B):
        for p in range(P):
            for q in range(Q):
                for r in range(R):
                    for s in range(S):
                        h, w = p * stride + r - pad, q * stride + s - pad
                        if 0 <= h < H and 0 <= w < Wd:
                            cols[(b * P + p) * Q + q, (r * S + s) * C_in:(r * S + s + 1) * C_in] = D[b, h, w]
    Wm = W.reshape(C_out, -1).astype(np.float64)
    assert np.allclose(oracle.conv_fwd(D, W, stride, pad)[0].reshape(-1, C_out), cols @ Wm.T, rtol=1e-12, atol=1e-12)
    Gm = G.reshape(-1, C_out).astype(np.float64)
    assert np.allclose(oracle.conv_bwd_weight(D, G, R, S, stride, pad)[0].reshape(C_out, -1), Gm.T @ cols, rtol=1e-12,
                       atol=1e-12)


@pytest.mark.parametrize("g", GEOMS)
def test_adjoint_identities_tie_the_three_products(g):
    B, H, Wd, C_in, C_out, R, S, stride, pad = g
    D, W, G = tensors(g, oracle.F32, seed=5)
    lhs = float(np.sum(oracle.conv_fwd(D, W, stride, pad)[0] * G))
    via_data = float(np.sum(oracle.conv_bwd_data(G, W, H, Wd, stride, pad)[0] * D))
    via_weight = float(np.sum(oracle.conv_bwd_weight(D, G, R, S, stride, pad)[0] * W))
    assert lhs == pytest.approx(via_data, rel=1e-11) and lhs == pytest.approx(via_weight, rel=1e-11)


def test_one_hot_filter_shifts_the_image():
    """W[k, r, s, c] = 1 alone: O[., p, q, k] = D[., p + r - pad, q + s - pad, c] (zero outside)."""
    D = wl.normal((1, 5, 6, 2), 1.0, 1, oracle.F32)
    for (r, s, c) in ((0, 0, 1), (2, 1, 0), (1, 2, 1)):
        W = np.zeros((1, 3, 3, 2), np.float32)
        W[0, r, s, c] = 1
        O = oracle.conv_fwd(D, W, 1, 1)[0]
        for p in range(5):
            for q in range(6):
                h, w = p + r - 1, q + s - 1
                want = D[0, h, w, c] if 0 <= h < 5 and 0 <= w < 6 else 0.0
                assert O[0, p, q, 0] == want


def test_sampled_outputs_equal_the_full_result():
    g = (2, 8, 8, 4, 6, 3, 3, 2, 1)
    D, W, G = tensors(g, oracle.BF16, seed=7)
    O, ab = oracle.conv_fwd(D, W, 2, 1)
    pix = np.array([0, 5, 17, O.shape[0] * O.shape[1] * O.shape[2] - 1])
    Os, abs_ = oracle.conv_fwd(D, W, 2, 1, pixels=pix)
    assert np.array_equal(Os, O.reshape(-1, 6)[pix]) and np.array_equal(abs_, ab.reshape(-1, 6)[pix])
    dW, ab = oracle.conv_bwd_weight(D, G, 3, 3, 2, 1)
    ent = np.array([0, 7, 100, dW.size - 1])
    dWs, abw = oracle.conv_bwd_weight(D, G, 3, 3, 2, 1, entries=ent)
    assert np.array_equal(dWs, dW.reshape(-1)[ent]) and np.array_equal(abw, ab.reshape(-1)[ent])
    with pytest.raises(ValueError):
        oracle.conv_fwd(D, W, 2, 1, pixels=np.array([O.size]))
    with pytest.raises(ValueError):
        oracle.conv_bwd_weight(D, G, 3, 3, 2, 1, entries=np.array([-1]))
