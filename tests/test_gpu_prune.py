"""GPU parity of sdgp_prune against the CPU oracle: bit-exact values, positions and dense-shaped output."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_00774_amd as sdgp
from paper_2202_00774_amd import workloads as wl
from util import to_gpu, to_host

pytestmark = pytest.mark.gpu

RANKERS = (oracle.RANDOM, oracle.GREEDY, oracle.GREEDY_ADJUSTED)
NM = [(2, 4), (2, 8), (2, 16), (1, 4), (1, 8), (3, 4), (4, 8), (4, 16), (8, 16), (2, 32), (4, 32), (16, 32), (4, 4),
      (3, 5), (2, 6), (1, 1), (2, 2), (5, 7), (8, 8)]


def check(dO_host, n, m, ranker, seed):
    ref_p, ref_v, ref_i = oracle.prune(dO_host, n, m, ranker, seed=seed)
    d = to_gpu(dO_host)
    before = d.clone()
    p, v, i = sdgp.sdgp_prune(d, n, m, ranker, seed, pruned=True, compact=True)
    torch.cuda.synchronize()
    assert torch.equal(d.view(torch.int16) if d.dtype == torch.bfloat16 else d.view(torch.int32),
                       before.view(torch.int16) if d.dtype == torch.bfloat16 else before.view(torch.int32))
    assert np.array_equal(to_host(i), ref_i)
    assert np.array_equal(to_host(p).view(np.uint8), ref_p.view(np.uint8))
    assert np.array_equal(to_host(v).view(np.uint8), ref_v.view(np.uint8))
    # each output alone gives the same bits
    p2, _, _ = sdgp.sdgp_prune(d, n, m, ranker, seed, pruned=True, compact=False)
    _, v3, i3 = sdgp.sdgp_prune(d, n, m, ranker, seed, pruned=False, compact=True)
    assert torch.equal(p2.view(torch.uint8), p.view(torch.uint8))
    assert torch.equal(v3.view(torch.uint8), v.view(torch.uint8)) and torch.equal(i3, i)


@pytest.mark.parametrize("ranker", RANKERS)
@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.F32])
@pytest.mark.parametrize("n,m", NM)
def test_prune_matches_oracle(ranker, dtype, n, m):
    # several blocks of 256 lanes plus a ragged tail; 30 % exact zeros make ties common
    rows, C = 37, m * 3 * 47
    dO = wl.laplace_with_zeros((rows, C), 1e-3, 0.3, seed=11 * m + n, dtype=dtype)
    check(dO, n, m, ranker, seed=12345 + m)


@pytest.mark.parametrize("ranker", RANKERS)
@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.F32])
def test_prune_tiny_and_odd_sizes(ranker, dtype):
    for rows, C, n, m in ((1, 4, 2, 4), (1, 8, 2, 4), (3, 12, 2, 4), (1, 16, 2, 16), (5, 8, 2, 8), (1, 32, 4, 32), (7, 20, 2, 4)):
        dO = wl.laplace_with_zeros((rows, C), 1.0, 0.4, seed=rows * 100 + C, dtype=dtype)
        check(dO, n, m, ranker, seed=7)


@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.F32])
def test_prune_special_values(dtype):
    """Signed zeros, subnormals, infinities and repeated magnitudes, in every position of a group."""
    if dtype == oracle.BF16:
        alphabet = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x3F80, 0xBF80, 0x7F80, 0xFF80, 0x7F7F, 0x4000],
                            np.uint16)
    else:
        alphabet = np.array([0.0, -0.0, 1e-45, -1e-45, 1.1754942e-38, 1.17549435e-38, 1.0, -1.0, np.inf, -np.inf,
                             3.4028235e38, 2.0], np.float32)
    rng = np.random.default_rng(3)
    dO = rng.choice(alphabet, size=(64, 256))
    for n, m in ((2, 4), (2, 8), (2, 16), (4, 8)):
        for ranker in (oracle.GREEDY, oracle.RANDOM):
            check(dO, n, m, ranker, seed=1)
    # the rescale is compared on finite data only (its result for infinite input is not defined by the method)
    finite = rng.choice(alphabet[:8] if dtype == oracle.BF16 else alphabet[:8], size=(64, 256))
    for n, m in ((2, 4), (2, 8), (2, 16)):
        check(finite, n, m, oracle.GREEDY_ADJUSTED, seed=1)


def test_prune_paper_example_on_gpu():
    d = torch.tensor([[1.0, 7.0, -3.0, 2.0]], device="cuda")
    p, v, i = sdgp.sdgp_prune(d, 2, 4, sdgp.GREEDY, compact=True)
    assert p.cpu().tolist() == [[0.0, 7.0, -3.0, 0.0]] and i.cpu().tolist() == [[1, 2]] and v.cpu().tolist() == [[7.0, -3.0]]


def test_prune_random_both_seed_words():
    """Both words of the seed matter."""
    dO = wl.laplace_with_zeros((16, 64), 1.0, 0.0, seed=1, dtype=oracle.BF16)
    for seed in (0, 1, 2 ** 32, 2 ** 63 + 5, 2 ** 64 - 1):
        check(dO, 2, 4, oracle.RANDOM, seed)


@pytest.mark.parametrize("n,m", [(2, 4), (2, 16)])
def test_prune_random_beyond_2_to_32_elements(n, m):
    """A tensor of 2^32 + 8192 bf16 elements: the high word of the flat element index enters the hash.  The rows around
    the 2^32 boundary and the last rows are compared with kept sets computed here from the oracle's hash of (seed, flat
    index): the n largest (key, -position) of every group; kept values are copies, dropped positions +0."""
    C = 64
    rows = (2 ** 32 + 8192) // C
    seed = 2 ** 33 + 12345
    d = torch.zeros((rows, C), dtype=torch.bfloat16, device="cuda")
    first = 2 ** 32 // C - 32                       # 32 rows below the boundary ... the end: 160 rows
    tail = wl.laplace_with_zeros((rows - first, C), 1.0, 0.0, seed=3, dtype=oracle.BF16)
    d[first:] = to_gpu(tail)
    p, _, _ = sdgp.sdgp_prune(d, n, m, sdgp.RANDOM, seed)
    got = to_host(p[first:])
    head = to_host(p[:64])
    del p, d
    want = np.zeros_like(tail)
    for r in range(tail.shape[0]):
        for g in range(C // m):
            e0 = (first + r) * C + g * m
            keys = [oracle.hash32(seed, e0 + j) for j in range(m)]
            order = sorted(range(m), key=lambda j: (-keys[j], j))[:n]
            for j in order:
                want[r, g * m + j] = tail[r, g * m + j]
    assert np.array_equal(got, want)
    assert not head.any()


@pytest.mark.parametrize("ranker", RANKERS)
def test_prune_resnet_sized_tensor(ranker):
    """A full config-2 gradient tensor (batch 512, 16x16, 256 channels = 33.5 M elements), compared in full."""
    dO = wl.laplace_with_zeros((512, 16, 16, 256), 1e-3, 0.3, seed=2003, dtype=oracle.BF16)
    ref_p, _, _ = oracle.prune(dO, 2, 4, ranker, seed=0)
    p, _, _ = sdgp.sdgp_prune(to_gpu(dO), 2, 4, ranker, 0)
    assert np.array_equal(to_host(p), ref_p)


def test_empty_tensor_is_a_noop():
    d = torch.empty((0, 16), dtype=torch.bfloat16, device="cuda")
    p, v, i = sdgp.sdgp_prune(d, 2, 4, sdgp.GREEDY, compact=True)
    assert p.shape == (0, 16) and v.shape == (0, 8)


def test_errors_raise():
    d = torch.zeros((2, 18), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sdgp.SdgpError):
        sdgp.sdgp_prune(d, 2, 4, sdgp.GREEDY)
    with pytest.raises(sdgp.SdgpError):
        sdgp.sdgp_prune(d, 3, 2, sdgp.GREEDY)
