"""Helpers shared by the tests: moving stored tensors between numpy (oracle side) and torch (GPU side)."""
import numpy as np
import torch


def to_gpu(a: np.ndarray) -> torch.Tensor:
    """uint16 arrays are bfloat16 bit patterns; float32 arrays go as they are."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def rel_error(got: np.ndarray, ref: np.ndarray, absum: np.ndarray) -> float:
    """max |got - ref| / sum_k |a_k||w_k|: the error of a sum of products relative to its condition scale."""
    return float(np.max(np.abs(got.astype(np.float64) - ref) / (absum + 1e-300)))
