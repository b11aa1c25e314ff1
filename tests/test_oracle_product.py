"""Pins for the CPU oracle's backward-data products (Fig. 1, Fig. 2, Fig. 3 of the paper).

Expectations come from a hand-worked example, from the library routines the
product reduces to when nothing is pruned (torch's fp64 matmul and the input
gradient of torch's conv2d), from an explicit im2col + matrix product written
here (Sec. II-A: convolution maps to a matrix product), and from the adjoint
identity <conv(D), G> = <D, conv_bwd_data(G)>.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_00774_amd import workloads as wl


def rand_storage(shape, seed, dtype, scale=1.0):
    return wl.normal(shape, scale, seed, dtype)


# --------------------------------------------------------------- linear

def test_hand_worked_linear_example():
    """Row [1,7,-3,2] against W rows [1,0],[0,1],[1,1],[2,-1]: dense gives [2,2]; 2:4 magnitude gives [-3,4]."""
    dO = np.array([[1, 7, -3, 2]], np.float32)
    W = np.array([[1, 0], [0, 1], [1, 1], [2, -1]], np.float32)
    dense, _ = oracle.linear_bwd_data(dO, W)
    assert dense.tolist() == [[2.0, 2.0]]
    pruned = oracle.prune(dO, 2, 4, oracle.GREEDY)[0]
    dD, ab = oracle.linear_bwd_data(pruned, W)
    assert dD.tolist() == [[-3.0, 4.0]]
    assert ab.tolist() == [[3.0, 10.0]]
    adj = oracle.prune(dO, 2, 4, oracle.GREEDY_ADJUSTED)[0]
    dD, _ = oracle.linear_bwd_data(adj, W)
    assert np.allclose(dD, [[-3.9, 5.2]], rtol=1e-6)


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_linear_dense_case_is_a_matrix_product(dtype):
    dO = rand_storage((37, 24), 1, dtype)
    W = rand_storage((24, 19), 2, dtype)
    kept_all = oracle.prune(dO, 4, 4, oracle.GREEDY)[0]
    dD, ab = oracle.linear_bwd_data(kept_all, W)
    a, w = torch.from_numpy(wl.to_f64(dO)), torch.from_numpy(wl.to_f64(W))
    assert np.allclose(dD, (a @ w).numpy(), rtol=1e-13, atol=1e-13)
    assert np.allclose(ab, (a.abs() @ w.abs()).numpy(), rtol=1e-13, atol=1e-13)


def test_linear_is_not_transposed():
    """W is [C_out, C_in]: a one-hot dO row k picks row k of W."""
    W = np.arange(12, dtype=np.float32).reshape(3, 4)
    for k in range(3):
        dO = np.zeros((1, 3), np.float32)
        dO[0, k] = 1
        assert oracle.linear_bwd_data(dO, W)[0][0].tolist() == W[k].tolist()


# ------------------------------------------------------------ convolution

def torch_conv_input_grad(dO, W, H, Wd, stride, pad):
    """Library special case: the input gradient of torch's conv2d (a cross-correlation) in fp64."""
    g = torch.from_numpy(wl.to_f64(dO)).permute(0, 3, 1, 2).contiguous()      # [B,K,P,Q]
    w = torch.from_numpy(wl.to_f64(W)).permute(0, 3, 1, 2).contiguous()       # [K,C,R,S]
    B = dO.shape[0]
    C = W.shape[3]
    x = torch.zeros((B, C, H, Wd), dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.conv2d(x, w, stride=stride, padding=pad)
    assert tuple(y.shape) == tuple(g.shape)
    y.backward(g)
    return x.grad.permute(0, 2, 3, 1).contiguous().numpy()                     # [B,H,W,C]


CONV_CASES = [
    # B, H, Wd, C_in, C_out, R, S, stride, pad
    (2, 6, 7, 5, 8, 3, 3, 1, 1),
    (1, 9, 8, 3, 4, 3, 3, 2, 1),
    (2, 11, 13, 3, 8, 7, 7, 2, 3),
    (2, 8, 6, 4, 8, 1, 1, 2, 0),
    (1, 5, 5, 6, 4, 1, 1, 1, 0),
    (1, 7, 6, 2, 4, 3, 2, 1, 0),
    (1, 10, 9, 2, 4, 5, 3, 3, 2),
    (3, 4, 4, 8, 8, 3, 3, 1, 1),
]


@pytest.mark.parametrize("case", CONV_CASES)
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_conv_dense_case_matches_library_input_gradient(case, dtype):
    B, H, Wd, C_in, C_out, R, S, stride, pad = case
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    dO = rand_storage((B, P, Q, C_out), 10, dtype)
    W = rand_storage((C_out, R, S, C_in), 11, dtype)
    dD, ab = oracle.conv_bwd_data(dO, W, H, Wd, stride, pad)
    want = torch_conv_input_grad(dO, W, H, Wd, stride, pad)
    assert dD.shape == want.shape
    assert np.allclose(dD, want, rtol=1e-12, atol=1e-12)
    # absum is the same product of magnitudes
    dOa = np.abs(wl.to_f64(dO)).astype(np.float32)
    Wa = np.abs(wl.to_f64(W)).astype(np.float32)
    if dtype == oracle.F32:
        want_ab = torch_conv_input_grad(dOa, Wa, H, Wd, stride, pad)
        assert np.allclose(ab, want_ab, rtol=1e-12, atol=1e-12)


def im2col_product(dOp, W, H, Wd, stride, pad):
    """Explicit im2col: build for every input pixel the row of all (tap, channel) gradient values, then one matrix product."""
    B, P, Q, K = dOp.shape
    _, R, S, C = W.shape
    g, w = wl.to_f64(dOp), wl.to_f64(W)
    cols = np.zeros((B, H, Wd, R, S, K))
    for h in range(H):
        for x in range(Wd):
            for r in range(R):
                for s in range(S):
                    hp, wq = h + pad - r, x + pad - s
                    if hp % stride or wq % stride:
                        continue
                    p, q = hp // stride, wq // stride
                    if 0 <= p < P and 0 <= q < Q:
                        cols[:, h, x, r, s, :] = g[:, p, q, :]
    wmat = w.transpose(1, 2, 0, 3).reshape(R * S * K, C)                      # [(r,s,k), c]
    return (cols.reshape(B * H * Wd, R * S * K) @ wmat).reshape(B, H, Wd, C)


@pytest.mark.parametrize("case", CONV_CASES[:4])
@pytest.mark.parametrize("ranker", [oracle.RANDOM, oracle.GREEDY, oracle.GREEDY_ADJUSTED])
def test_pruned_conv_equals_im2col_product(case, ranker):
    B, H, Wd, C_in, C_out, R, S, stride, pad = case
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    dO = wl.laplace_with_zeros((B, P, Q, C_out), 1e-3, 0.3, seed=20, dtype=oracle.BF16)
    W = rand_storage((C_out, R, S, C_in), 21, oracle.BF16, 0.1)
    pruned = oracle.prune(dO, 2, 4, ranker, seed=4)[0]
    dD, _ = oracle.conv_bwd_data(pruned, W, H, Wd, stride, pad)
    assert np.allclose(dD, im2col_product(pruned, W, H, Wd, stride, pad), rtol=1e-12, atol=1e-18)


def test_one_by_one_conv_is_the_linear_product():
    dO = rand_storage((2, 5, 4, 16), 30, oracle.BF16)
    W = rand_storage((16, 1, 1, 12), 31, oracle.BF16)
    pruned = oracle.prune(dO, 2, 8, oracle.GREEDY)[0]
    conv, cab = oracle.conv_bwd_data(pruned, W, 5, 4, 1, 0)
    lin, lab = oracle.linear_bwd_data(pruned.reshape(40, 16), W.reshape(16, 12))
    assert np.array_equal(conv.reshape(40, 12), lin) and np.array_equal(cab.reshape(40, 12), lab)


def forward_conv(D, W, stride, pad):
    """Cross-correlation forward pass written out (test-only), fp64, NHWC / KRSC."""
    B, H, Wd, C = D.shape
    K, R, S, _ = W.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    Dp = np.zeros((B, H + 2 * pad, Wd + 2 * pad, C))
    Dp[:, pad:pad + H, pad:pad + Wd] = D
    O = np.zeros((B, P, Q, K))
    for p in range(P):
        for q in range(Q):
            patch = Dp[:, p * stride:p * stride + R, q * stride:q * stride + S, :]      # [B,R,S,C]
            O[:, p, q, :] = np.einsum("brsc,krsc->bk", patch, W)
    return O


@pytest.mark.parametrize("case", CONV_CASES)
def test_adjoint_identity(case):
    """<forward(D), G> == <D, backward_data(G)> for every D: backward-data is the transpose of the forward map."""
    B, H, Wd, C_in, C_out, R, S, stride, pad = case
    rng = np.random.default_rng(5)
    D = rng.standard_normal((B, H, Wd, C_in))
    W = rand_storage((C_out, R, S, C_in), 41, oracle.F32)
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    G = rand_storage((B, P, Q, C_out), 42, oracle.F32)
    lhs = float((forward_conv(D, W.astype(np.float64), stride, pad) * G).sum())
    rhs = float((D * oracle.conv_bwd_data(G, W, H, Wd, stride, pad)[0]).sum())
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))


def test_strided_one_by_one_leaves_untouched_pixels_zero():
    dO = rand_storage((1, 3, 3, 4), 50, oracle.F32)
    W = rand_storage((4, 1, 1, 2), 51, oracle.F32)
    dD, _ = oracle.conv_bwd_data(dO, W, 6, 6, 2, 0)
    mask = np.zeros((6, 6), bool)
    mask[::2, ::2] = True
    assert np.all(dD[0][~mask] == 0) and np.all(dD[0][mask].any(axis=-1))


def test_sampled_pixels_equal_full_result():
    B, H, Wd, C_in, C_out = 2, 9, 7, 6, 8
    dO = wl.laplace_with_zeros((B, H, Wd, C_out), 1e-3, 0.3, seed=60, dtype=oracle.BF16)
    W = rand_storage((C_out, 3, 3, C_in), 61, oracle.BF16, 0.1)
    pruned = oracle.prune(dO, 2, 4, oracle.GREEDY)[0]
    full, fab = oracle.conv_bwd_data(pruned, W, H, Wd, 1, 1)
    pix = np.array([0, 6, 62, 63, 125, 17], np.int64)
    part, pab = oracle.conv_bwd_data(pruned, W, H, Wd, 1, 1, pixels=pix)
    assert np.array_equal(part, full.reshape(-1, C_in)[pix]) and np.array_equal(pab, fab.reshape(-1, C_in)[pix])


def test_fp64_against_fp32_accumulation_brackets_the_tolerance():
    """An fp32-accumulating product of the config-1 shapes stays far inside the 1e-5 bound relative to absum."""
    dO, W = wl.linear_config1()
    pruned = oracle.prune(dO, 2, 4, oracle.GREEDY)[0]
    dD, ab = oracle.linear_bwd_data(pruned, W)
    acc = np.zeros((256, 256), np.float32)
    for k in range(128):
        acc += pruned[:, k:k + 1] * W[k:k + 1, :]
    err = np.abs(acc.astype(np.float64) - dD) / (ab + 1e-300)
    assert err.max() < 1e-5 / 4
