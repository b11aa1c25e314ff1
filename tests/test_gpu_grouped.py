"""GPU parity of the grouped backward-data product (Sec. IV: RegNetX's group convolutions) against the oracle.

Tolerance as for the ungrouped product: 1e-2 (bf16) / 1e-5 (fp32) of the sum of |a||b| over an element's terms.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_00774_amd as sdgp
from paper_2202_00774_amd import workloads as wl
from util import to_gpu, to_host

pytestmark = pytest.mark.gpu

# B, H, Wd, C_in, C_out, R, S, stride, pad, groups
GEOMS = [
    (3, 14, 14, 48, 48, 3, 3, 1, 1, 3),        # group width 16 as in RegNetX-400MF: the matrix-core kernel (bf16)
    (2, 20, 37, 160, 160, 3, 3, 1, 1, 10),     # the same kernel: ragged tiles both ways, a slab of two groups
    (5, 7, 7, 64, 64, 3, 3, 1, 1, 4),          # images smaller than a tile
    (2, 15, 13, 64, 64, 3, 3, 2, 1, 4),        # the stride-2 block of a stage: four parity classes, odd image sizes
    (3, 28, 70, 160, 160, 3, 3, 2, 1, 10),     # stride 2, even sizes, two column tiles, a slab of two groups
    (2, 9, 9, 32, 64, 1, 1, 1, 0, 2),
    (2, 8, 8, 16, 16, 3, 3, 1, 1, 4),          # four channels per group: one 2:4 group each
    (1, 12, 10, 24, 48, 5, 3, 1, 1, 3),
]
RANKERS = [oracle.RANDOM, oracle.GREEDY, oracle.GREEDY_ADJUSTED]


def run(geom, dtype, n, m, ranker, seed):
    B, H, Wd, C_in, C_out, R, S, stride, pad, groups = geom
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(Wd, S, stride, pad)
    dO = wl.laplace_with_zeros((B, P, Q, C_out), 1e-3, 0.3, 7 + C_out, dtype)
    W = wl.normal((C_out, R, S, C_in // groups), 0.1, 8 + C_in, dtype)
    pruned = oracle.prune(dO, n, m, ranker, seed=seed)[0]
    ref, ab = oracle.conv_bwd_data_grouped(pruned, W, H, Wd, stride, pad, groups)
    out = sdgp.sdgp_conv_bwd_data_grouped(to_gpu(dO), to_gpu(W), H, Wd, stride, pad, groups, n, m, ranker, seed)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (B, H, Wd, C_in)
    got = wl.to_f64(to_host(out))
    err = np.abs(got - ref) / (ab + 1e-300)
    tol = 1e-2 if dtype == oracle.BF16 else 1e-5
    assert np.all(got[ab == 0] == 0)
    assert err[ab > 0].max() <= tol, (geom, n, m, ranker, err.max())


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("ranker", RANKERS)
@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.F32])
def test_grouped_matches_oracle(geom, ranker, dtype):
    for n, m in ((2, 4), (4, 4), (1, 4)):
        run(geom, dtype, n, m, ranker, 3)
    if (geom[4] // geom[9]) % 16 == 0:
        run(geom, dtype, 2, 16, ranker, 4)
        run(geom, dtype, 4, 8, ranker, 5)


def test_one_group_is_the_ungrouped_call():
    L = wl.ConvLayer("g1", 2, 10, 10, 32, 64, 3, 3, 1, 1)
    dO, W = wl.layer_inputs(L, 1e-3, 0.3, seed=5, dtype=oracle.BF16)
    a = sdgp.sdgp_conv_bwd_data_grouped(to_gpu(dO), to_gpu(W), 10, 10, 1, 1, 1, 2, 4, sdgp.GREEDY, 0)
    b = sdgp.sdgp_conv_bwd_data(to_gpu(dO), to_gpu(W), 10, 10, 1, 1, 2, 4, sdgp.GREEDY, 0)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_groups_that_split_an_m_group_are_refused():
    dO = torch.zeros((1, 4, 4, 8), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((8, 3, 3, 2), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sdgp.SdgpError):
        sdgp.sdgp_conv_bwd_data_grouped(dO, W, 4, 4, 1, 1, 4, 2, 4, sdgp.GREEDY)     # two output channels per group, m = 4
    with pytest.raises(sdgp.SdgpError):
        sdgp.sdgp_conv_bwd_data_grouped(dO, W, 4, 4, 1, 1, 3, 4, 4, sdgp.GREEDY)     # 8 % 3 != 0


def test_group_width_16_keeps_exactly_the_oracle_values():
    """The matrix-core kernel for 16-channel groups prunes in LDS: with a one-hot filter (output channel k feeds input
    channel k through the centre tap) dD must equal the oracle's pruned gradient bit for bit."""
    B, H, Wd, C, groups = 3, 19, 33, 96, 6
    dO = wl.laplace_with_zeros((B, H, Wd, C), 1e-3, 0.3, 77, wl.BF16)
    W = np.zeros((C, 3, 3, 16), np.uint16)
    for k in range(C):
        W[k, 1, 1, k % 16] = 0x3F80
    d, w = to_gpu(dO), to_gpu(W)
    for n, m, ranker in ((2, 4, oracle.RANDOM), (2, 4, oracle.GREEDY), (2, 4, oracle.GREEDY_ADJUSTED), (1, 4, oracle.GREEDY),
                         (2, 8, oracle.RANDOM), (2, 8, oracle.GREEDY_ADJUSTED), (2, 16, oracle.GREEDY), (2, 16, oracle.RANDOM),
                         (4, 8, oracle.GREEDY), (4, 16, oracle.GREEDY_ADJUSTED), (3, 4, oracle.RANDOM), (16, 16, oracle.GREEDY)):
        want = oracle.prune(dO, n, m, ranker, seed=9)[0]
        got = to_host(sdgp.sdgp_conv_bwd_data_grouped(d, w, H, Wd, 1, 1, groups, n, m, ranker, 9))
        torch.cuda.synchronize()
        a, b = wl.to_f64(got), wl.to_f64(want)          # (a kept -0 may come out as +0: compare values)
        assert np.array_equal(a, b), (n, m, ranker, int(np.count_nonzero(a != b)))


def test_group_width_16_stride_2_keeps_exactly_the_oracle_values():
    """The same through the stride-2 form of the kernel: the centre tap of output pixel (p, q) read input pixel
    (2p, 2q), so dD there equals the pruned gradient and every other input pixel receives nothing."""
    B, H, Wd, C, groups = 2, 21, 38, 64, 4
    P, Q = (H - 1) // 2 + 1, (Wd - 1) // 2 + 1
    dO = wl.laplace_with_zeros((B, P, Q, C), 1e-3, 0.3, 78, wl.BF16)
    W = np.zeros((C, 3, 3, 16), np.uint16)
    for k in range(C):
        W[k, 1, 1, k % 16] = 0x3F80
    d, w = to_gpu(dO), to_gpu(W)
    for n, m, ranker in ((2, 4, oracle.RANDOM), (2, 4, oracle.GREEDY_ADJUSTED), (2, 8, oracle.GREEDY), (2, 16, oracle.RANDOM),
                         (4, 16, oracle.GREEDY), (4, 4, oracle.GREEDY)):
        want = wl.to_f64(oracle.prune(dO, n, m, ranker, seed=3)[0])
        got = wl.to_f64(to_host(sdgp.sdgp_conv_bwd_data_grouped(d, w, H, Wd, 2, 1, groups, n, m, ranker, 3)))
        torch.cuda.synchronize()
        assert np.array_equal(got[:, ::2, ::2, :], want), (n, m, ranker)
        rest = got.copy()
        rest[:, ::2, ::2, :] = 0
        assert not rest.any()
