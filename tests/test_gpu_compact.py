"""GPU parity of the compacted-gradient backward-data path (K' = (n/m) C_out kept values per pixel, W rows gathered by
index; Sec. III-A, Sec. IV-C) against the oracle: prune, then the plain backward-data sum.  Tolerance as for the fused
path: |gpu - ref| <= 1e-2 * sum |a||w| (bf16 inputs, fp32 accumulation, one bf16 rounding of the result)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_00774_amd as sdgp
from paper_2202_00774_amd import workloads as wl
from util import to_gpu, to_host

pytestmark = pytest.mark.gpu

LAYERS = [
    wl.ConvLayer("pw_64x256", 3, 23, 21, 64, 256, 1, 1, 1, 0),          # 8 lanes per pixel, ragged last workgroup
    wl.ConvLayer("pw_256x64", 2, 14, 14, 256, 64, 1, 1, 1, 0),          # 32 lanes per pixel
    wl.ConvLayer("pw_520x96", 1, 9, 11, 520, 96, 1, 1, 1, 0),           # two channel blocks, the second partly empty
    wl.ConvLayer("c3_128x256", 2, 16, 16, 128, 256, 3, 3, 1, 1),        # filter in several LDS chunks
    wl.ConvLayer("c3_s2_64x128", 2, 15, 17, 64, 128, 3, 3, 2, 1),       # stride 2: taps that reach no gradient pixel
    wl.ConvLayer("c5_40x64", 1, 10, 10, 40, 64, 5, 5, 1, 2),
    wl.ConvLayer("linear_1000", 257, 1, 1, 512, 1024, 1, 1, 1, 0),
]
SETTINGS = [(2, 16, oracle.GREEDY), (4, 32, oracle.GREEDY), (2, 32, oracle.GREEDY_ADJUSTED), (2, 4, oracle.RANDOM),
            (1, 8, oracle.GREEDY), (8, 8, oracle.GREEDY)]


@pytest.mark.parametrize("L", LAYERS, ids=lambda L: L.name)
def test_compact_path_matches_oracle(L):
    dO, W = wl.layer_inputs(L, 1e-3, 0.3, seed=77 + L.C_out, dtype=wl.BF16)
    d, w = to_gpu(dO), to_gpu(W)
    for n, m, rk in SETTINGS:
        if L.C_out % m:
            continue
        pruned = oracle.prune(dO, n, m, rk, seed=5)[0]
        ref, ab = oracle.conv_bwd_data(pruned, W, L.H, L.Wd, L.stride, L.pad)
        out = sdgp.sdgp_conv_bwd_data_compact(d, w, L.H, L.Wd, L.stride, L.pad, n, m, rk, 5)
        torch.cuda.synchronize()
        got = wl.to_f64(to_host(out))
        assert np.all(got[ab == 0] == 0), (L.name, n, m)
        err = np.abs(got - ref) / (ab + 1e-300)
        assert err[ab > 0].max() <= 1e-2, (L.name, n, m, rk, err.max())


def test_compact_path_at_bench_size_sampled():
    """64 <- 256 channels at 56 x 56, batch 128 (an HBM-bound ResNet-50 layer), 2:16: sampled pixels."""
    L = wl.resnet50_bottleneck_layers(128)[2]
    dO, W = wl.layer_inputs(L, 1e-4, 0.4, seed=3002, dtype=wl.BF16)
    pixels = np.unique(np.concatenate([[0, L.B * L.H * L.Wd - 1], np.random.default_rng(1).integers(0, L.B * L.H * L.Wd, 4000)]))
    pruned = oracle.prune(dO, 2, 16, oracle.GREEDY, seed=0)[0]
    ref, ab = oracle.conv_bwd_data(pruned, W, L.H, L.Wd, L.stride, L.pad, pixels=pixels)
    out = sdgp.sdgp_conv_bwd_data_compact(to_gpu(dO), to_gpu(W), L.H, L.Wd, L.stride, L.pad, 2, 16, sdgp.GREEDY, 0)
    torch.cuda.synchronize()
    got = wl.to_f64(to_host(out.reshape(-1, L.C_in)[torch.from_numpy(pixels).cuda()]))
    assert (np.abs(got - ref) / (ab + 1e-300))[ab > 0].max() <= 1e-2


def test_compact_path_refuses_what_it_does_not_take():
    d = torch.zeros((1, 4, 4, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sdgp.SdgpError):   # C_in not a multiple of 8
        sdgp.sdgp_conv_bwd_data_compact(d, torch.zeros((16, 1, 1, 12), dtype=torch.bfloat16, device="cuda"), 4, 4, 1, 0, 2, 4, sdgp.GREEDY)
    with pytest.raises(sdgp.SdgpError):   # fp32
        sdgp.sdgp_conv_bwd_data_compact(d.float(), torch.zeros((16, 1, 1, 8), device="cuda"), 4, 4, 1, 0, 2, 4, sdgp.GREEDY)
    empty = sdgp.sdgp_conv_bwd_data_compact(torch.zeros((0, 4, 4, 16), dtype=torch.bfloat16, device="cuda"),
                                            torch.zeros((16, 1, 1, 8), dtype=torch.bfloat16, device="cuda"), 4, 4, 1, 0, 2, 4, sdgp.GREEDY)
    assert empty.shape == (0, 4, 4, 8)
