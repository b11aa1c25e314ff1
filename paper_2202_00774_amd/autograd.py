"""Drop-in autograd functions: the data gradient of a convolution or linear layer goes through the library.

SDGP prunes only the gradient that flows back to the earlier layers (Sec. III-A, Fig. 1): the weight gradient is
computed from the dense output gradient, which is why dL/dO is never modified.  Forward and weight gradient are
PyTorch's own kernels (outside this library's path); ``backward`` hands dL/dO (NHWC) and the weights (KRSC) to
``sdgp_conv_bwd_data`` / ``sdgp_linear_bwd_data`` and returns what they compute.  bf16 CUDA tensors.

    y = sdgp_conv2d(x, weight, stride=1, padding=1, n=2, m=4, ranker=GREEDY, seed=step)
    y = sdgp_linear(x, weight, n=2, m=4, ranker=GREEDY_ADJUSTED)

``n == m`` gives the dense data gradient from the same kernels.  ``per_channel=True`` selects the second reading of
Rescaled Magnitude (Sec. III-B figure captions): Magnitude pruning with one rescaling factor per output channel taken
over the whole gradient tensor; ``ranker`` and ``seed`` are then not used.
"""
from __future__ import annotations

import torch
import torch.nn.functional as F

from . import binding


class _Conv2dFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, stride, padding, n, m, ranker, seed, per_channel, groups):
        ctx.save_for_backward(x, weight)
        ctx.cfg = (int(stride), int(padding), int(n), int(m), int(ranker), int(seed), bool(per_channel), int(groups))
        return F.conv2d(x, weight, None, stride, padding, 1, int(groups))

    @staticmethod
    def backward(ctx, gy):
        x, weight = ctx.saved_tensors
        stride, padding, n, m, ranker, seed, per_channel, groups = ctx.cfg
        gx = gw = None
        if ctx.needs_input_grad[1]:
            gw = torch.nn.grad.conv2d_weight(x, weight.shape, gy, stride, padding, 1, groups)  # dense dL/dO
        if ctx.needs_input_grad[0]:
            dO = gy.permute(0, 2, 3, 1).contiguous()          # [B, P, Q, C_out]; a view when gy is channels_last
            Wk = weight.permute(0, 2, 3, 1).contiguous()      # [C_out, R, S, C_in]
            if groups > 1:
                dD = binding.sdgp_conv_bwd_data_grouped(dO, Wk, x.shape[2], x.shape[3], stride, padding, groups, n, m, ranker, seed)
            elif per_channel:
                dD = binding.sdgp_conv_bwd_data_channel_rescaled(dO, Wk, x.shape[2], x.shape[3], stride, padding, n, m)
            else:
                dD = binding.sdgp_conv_bwd_data(dO, Wk, x.shape[2], x.shape[3], stride, padding, n, m, ranker, seed)
            gx = dD.permute(0, 3, 1, 2)                       # NCHW view of NHWC memory (channels_last)
        return gx, gw, None, None, None, None, None, None, None, None


class _LinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, n, m, ranker, seed, per_channel):
        ctx.save_for_backward(x, weight)
        ctx.cfg = (int(n), int(m), int(ranker), int(seed), bool(per_channel))
        return F.linear(x, weight)

    @staticmethod
    def backward(ctx, gy):
        x, weight = ctx.saved_tensors
        n, m, ranker, seed, per_channel = ctx.cfg
        gx = gw = None
        g2 = gy.reshape(-1, gy.shape[-1])
        if ctx.needs_input_grad[1]:
            gw = g2.t() @ x.reshape(-1, x.shape[-1])          # dense dL/dO
        if ctx.needs_input_grad[0]:
            if per_channel:
                gx = binding.sdgp_linear_bwd_data_channel_rescaled(g2.contiguous(), weight.contiguous(), n, m).reshape(x.shape)
            else:
                gx = binding.sdgp_linear_bwd_data(g2.contiguous(), weight.contiguous(), n, m, ranker, seed).reshape(x.shape)
        return gx, gw, None, None, None, None, None


def sdgp_conv2d(x: torch.Tensor, weight: torch.Tensor, stride: int = 1, padding: int = 0, n: int = 2, m: int = 4,
                ranker: int = binding.GREEDY, seed: int = 0, per_channel: bool = False, groups: int = 1) -> torch.Tensor:
    """conv2d (no bias, dilation 1; x [B,C,H,W], weight [K,C/groups,R,S]) whose input gradient is SDGP-pruned.
    With groups > 1 (K/groups a multiple of m) the per-channel reading of the rescale is not available."""
    if groups > 1 and per_channel:
        raise ValueError("per_channel is not available for grouped convolutions")
    return _Conv2dFn.apply(x, weight, stride, padding, n, m, ranker, seed, per_channel, groups)


def sdgp_linear(x: torch.Tensor, weight: torch.Tensor, n: int = 2, m: int = 4, ranker: int = binding.GREEDY,
                seed: int = 0, per_channel: bool = False) -> torch.Tensor:
    """x @ weight.T (x [..., in], weight [out, in]) whose input gradient is SDGP-pruned along the `out` axis."""
    return _LinearFn.apply(x, weight, n, m, ranker, seed, per_channel)
