"""The autograd wrappers hand the right tensors to the library: input gradients against the oracle, weight gradients
against PyTorch's dense ones."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_00774_amd as sdgp
from paper_2202_00774_amd import autograd as sa
from paper_2202_00774_amd import workloads as wl

pytestmark = pytest.mark.gpu


def bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def rel_error(got, ref, ab):
    return float(np.max(np.abs(got - ref) / (ab + 1e-30)))


@pytest.mark.parametrize("stride,pad,R", [(1, 1, 3), (2, 1, 3), (1, 0, 1)])
@pytest.mark.parametrize("n,m,ranker", [(2, 4, sdgp.GREEDY), (2, 8, sdgp.RANDOM), (4, 4, sdgp.GREEDY)])
def test_conv2d_gradients(stride, pad, R, n, m, ranker):
    torch.manual_seed(3)
    B, C, K, H = 6, 16, 32, 13
    x = torch.randn(B, C, H, H, device="cuda", dtype=torch.bfloat16).contiguous(memory_format=torch.channels_last).requires_grad_()
    w = (torch.randn(K, C, R, R, device="cuda", dtype=torch.bfloat16) * 0.2).requires_grad_()
    y = sa.sdgp_conv2d(x, w, stride, pad, n, m, ranker, seed=11)
    gy = (torch.randn_like(y) * 1e-2).contiguous(memory_format=torch.channels_last)
    y.backward(gy)
    # weight gradient: PyTorch's own, from the dense gradient
    xr = x.detach().clone().requires_grad_()
    wr = w.detach().clone().requires_grad_()
    torch.nn.functional.conv2d(xr, wr, None, stride, pad).backward(gy)
    assert torch.allclose(w.grad.float(), wr.grad.float(), rtol=2e-2, atol=2e-2 * wr.grad.float().abs().max().item())
    # input gradient: prune(dO) x W by the oracle
    dO = bits(gy.permute(0, 2, 3, 1))
    Wk = bits(w.permute(0, 2, 3, 1))
    pruned = oracle.prune(dO, n, m, ranker, seed=11)[0]
    ref, ab = oracle.conv_bwd_data(pruned, Wk, H, H, stride, pad)
    got = wl.to_f64(bits(x.grad.permute(0, 2, 3, 1)))
    assert rel_error(got, ref, ab) <= 1e-2
    if n == m:  # the dense product is also PyTorch's input gradient
        assert torch.allclose(x.grad.float(), xr.grad.float(), rtol=3e-2, atol=3e-2 * xr.grad.float().abs().max().item())


def test_linear_gradients():
    torch.manual_seed(4)
    x = torch.randn(5, 40, 24, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    w = (torch.randn(64, 24, device="cuda", dtype=torch.bfloat16) * 0.2).requires_grad_()
    y = sa.sdgp_linear(x, w, 2, 4, sdgp.GREEDY_ADJUSTED, seed=2)
    gy = torch.randn_like(y) * 1e-2
    y.backward(gy)
    dO = bits(gy.reshape(-1, 64))
    pruned = oracle.prune(dO, 2, 4, oracle.GREEDY_ADJUSTED, seed=2)[0]
    ref, ab = oracle.linear_bwd_data(pruned, bits(w))
    assert rel_error(wl.to_f64(bits(x.grad.reshape(-1, 24))), ref, ab) <= 1e-2
    gw_ref = gy.reshape(-1, 64).float().t() @ x.detach().reshape(-1, 24).float()
    assert torch.allclose(w.grad.float(), gw_ref, rtol=2e-2, atol=2e-2 * gw_ref.abs().max().item())


def test_per_channel_rescale_through_autograd():
    torch.manual_seed(5)
    B, C, K, H = 6, 16, 32, 13
    x = torch.randn(B, C, H, H, device="cuda", dtype=torch.bfloat16).contiguous(memory_format=torch.channels_last).requires_grad_()
    w = (torch.randn(K, C, 3, 3, device="cuda", dtype=torch.bfloat16) * 0.2).requires_grad_()
    y = sa.sdgp_conv2d(x, w, 1, 1, 2, 4, per_channel=True)
    gy = (torch.randn_like(y) * 1e-2).contiguous(memory_format=torch.channels_last)
    y.backward(gy)
    dO = bits(gy.permute(0, 2, 3, 1))
    pruned = oracle.prune_channel_rescaled(dO.reshape(-1, K), 2, 4)[0].reshape(dO.shape)
    ref, ab = oracle.conv_bwd_data(pruned, bits(w.permute(0, 2, 3, 1)), H, H, 1, 1)
    assert rel_error(wl.to_f64(bits(x.grad.permute(0, 2, 3, 1))), ref, ab) <= 1e-2
    wr = w.detach().clone().requires_grad_()
    torch.nn.functional.conv2d(x.detach(), wr, None, 1, 1).backward(gy)
    assert torch.allclose(w.grad.float(), wr.grad.float(), rtol=2e-2, atol=2e-2 * wr.grad.float().abs().max().item())

    xl = torch.randn(7, 30, 24, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    wl_ = (torch.randn(64, 24, device="cuda", dtype=torch.bfloat16) * 0.2).requires_grad_()
    yl = sa.sdgp_linear(xl, wl_, 2, 4, per_channel=True)
    gl = torch.randn_like(yl) * 1e-2
    yl.backward(gl)
    pruned = oracle.prune_channel_rescaled(bits(gl.reshape(-1, 64)), 2, 4)[0]
    ref, ab = oracle.linear_bwd_data(pruned, bits(wl_))
    assert rel_error(wl.to_f64(bits(xl.grad.reshape(-1, 24))), ref, ab) <= 1e-2


@pytest.mark.parametrize("groups,stride", [(4, 1), (2, 2)])
def test_grouped_conv2d_gradients(groups, stride):
    """A grouped layer (RegNetX style): input gradient against the grouped oracle, weight gradient PyTorch's."""
    torch.manual_seed(6)
    B, C, K, H = 4, 32, 64, 12
    x = torch.randn(B, C, H, H, device="cuda", dtype=torch.bfloat16).contiguous(memory_format=torch.channels_last).requires_grad_()
    w = (torch.randn(K, C // groups, 3, 3, device="cuda", dtype=torch.bfloat16) * 0.2).requires_grad_()
    y = sa.sdgp_conv2d(x, w, stride, 1, 2, 4, sdgp.GREEDY_ADJUSTED, seed=0, groups=groups)
    gy = (torch.randn_like(y) * 1e-2).contiguous(memory_format=torch.channels_last)
    y.backward(gy)
    xr, wr = x.detach().clone().requires_grad_(), w.detach().clone().requires_grad_()
    torch.nn.functional.conv2d(xr, wr, None, stride, 1, 1, groups).backward(gy)
    assert torch.allclose(w.grad.float(), wr.grad.float(), rtol=2e-2, atol=2e-2 * wr.grad.float().abs().max().item())
    pruned = oracle.prune(bits(gy.permute(0, 2, 3, 1)), 2, 4, oracle.GREEDY_ADJUSTED)[0]
    ref, ab = oracle.conv_bwd_data_grouped(pruned, bits(w.permute(0, 2, 3, 1)), H, H, stride, 1, groups)
    assert rel_error(wl.to_f64(bits(x.grad.permute(0, 2, 3, 1))), ref, ab) <= 1e-2
    with pytest.raises(ValueError):
        sa.sdgp_conv2d(x, w, stride, 1, 2, 4, groups=groups, per_channel=True)
