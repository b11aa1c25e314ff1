"""ctypes binding of libsdgp.so: argument marshalling only.

Every function takes torch tensors that live on the GPU, hands their device
pointers and the current HIP stream to the C ABI, and raises ``SdgpError`` on a
non-zero status.  PyTorch is used for device memory and streams, nothing else.
"""
from __future__ import annotations

import ctypes
import os
import threading

import torch

F32, BF16 = 0, 1
RANDOM, GREEDY, GREEDY_ADJUSTED = 0, 1, 2

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libsdgp.so")
_lock = threading.Lock()
_lib = None

EXPORTS = ("sdgp_prune", "sdgp_linear_bwd_data", "sdgp_conv_bwd_data", "sdgp_conv_bwd_data_workspace",
           "sdgp_status_string", "sdgp_version")


class SdgpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where} failed with status {status}: {status_string(status)}")


def library_path() -> str:
    return _LIB_PATH


def load():
    """Loads libsdgp.so; raises if it has not been built (there is no fallback)."""
    global _lib
    with _lock:
        if _lib is None:
            if not os.path.exists(_LIB_PATH):
                raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2202_00774_amd.build`")
            lib = ctypes.CDLL(_LIB_PATH)
            i64, u64, i32, vp, sz = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
            lib.sdgp_prune.restype = i32
            lib.sdgp_prune.argtypes = [vp, i64, i64, i32, i32, i32, i32, u64, vp, vp, vp, vp]
            lib.sdgp_linear_bwd_data.restype = i32
            lib.sdgp_linear_bwd_data.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, u64, vp]
            lib.sdgp_conv_bwd_data.restype = i32
            lib.sdgp_conv_bwd_data.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32, i32,
                                               i32, u64, vp, sz, vp]
            lib.sdgp_conv_bwd_data_workspace.restype = sz
            lib.sdgp_conv_bwd_data_workspace.argtypes = [i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32, i32]
            lib.sdgp_status_string.restype = ctypes.c_char_p
            lib.sdgp_status_string.argtypes = [i32]
            lib.sdgp_version.restype = i32
            lib.sdgp_version.argtypes = []
            _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().sdgp_status_string(int(status)).decode()


def version() -> int:
    return int(load().sdgp_version())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}: float32 or bfloat16")


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def sdgp_prune(dO: torch.Tensor, n: int, m: int, ranker: int, seed: int = 0, *, pruned: bool = True,
               compact: bool = False):
    """Alg. 1 on ``dO`` ([..., C], channels last).  Returns ``(pruned, vals, idx)``; entries not asked for are None."""
    _dev(dO, "dO")
    C = dO.shape[-1]
    rows = dO.numel() // C if C else 0
    out = torch.empty_like(dO) if pruned else None
    vals = idx = None
    if compact:
        if m < 1 or C % m:
            raise SdgpError(-3, "sdgp_prune")
        kshape = tuple(dO.shape[:-1]) + (C // m * n,)
        vals = torch.empty(kshape, dtype=dO.dtype, device=dO.device)
        idx = torch.empty(kshape, dtype=torch.uint8, device=dO.device)
    rc = load().sdgp_prune(_ptr(dO), rows, C, _dtype_code(dO), n, m, ranker, seed & (2**64 - 1), _ptr(out),
                           _ptr(vals), _ptr(idx), _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_prune")
    return out, vals, idx


def sdgp_linear_bwd_data(dO: torch.Tensor, W: torch.Tensor, n: int, m: int, ranker: int, seed: int = 0,
                         out: torch.Tensor | None = None) -> torch.Tensor:
    """dD = prune(dO) @ W for dO [rows, C_out], W [C_out, C_in]."""
    _dev(dO, "dO"), _dev(W, "W")
    if dO.dim() != 2 or W.dim() != 2 or W.shape[0] != dO.shape[1] or W.dtype != dO.dtype:
        raise ValueError("expected dO [rows, C_out] and W [C_out, C_in] of one dtype")
    rows, C_out = dO.shape
    C_in = W.shape[1]
    if out is None:
        out = torch.empty((rows, C_in), dtype=dO.dtype, device=dO.device)
    _dev(out, "out")
    rc = load().sdgp_linear_bwd_data(_ptr(dO), _ptr(W), _ptr(out), rows, C_out, C_in, _dtype_code(dO), n, m, ranker,
                                     seed & (2**64 - 1), _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_linear_bwd_data")
    return out


def conv_bwd_data_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dtype_code, n, m) -> int:
    return int(load().sdgp_conv_bwd_data_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dtype_code, n, m))


def sdgp_conv_bwd_data(dO: torch.Tensor, W: torch.Tensor, H: int, Wd: int, stride: int, pad: int, n: int, m: int,
                       ranker: int, seed: int = 0, out: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None) -> torch.Tensor:
    """dD [B,H,Wd,C_in] from dO [B,P,Q,C_out] (NHWC) and W [C_out,R,S,C_in]."""
    _dev(dO, "dO"), _dev(W, "W")
    if dO.dim() != 4 or W.dim() != 4 or W.shape[0] != dO.shape[3] or W.dtype != dO.dtype:
        raise ValueError("expected dO [B,P,Q,C_out] and W [C_out,R,S,C_in] of one dtype")
    B, P, Q, C_out = dO.shape
    _, R, S, C_in = W.shape
    if (H + 2 * pad - R) // stride + 1 != P or (Wd + 2 * pad - S) // stride + 1 != Q:
        raise ValueError("dO's spatial size does not match H, Wd, stride, pad")
    if out is None:
        out = torch.empty((B, H, Wd, C_in), dtype=dO.dtype, device=dO.device)
    _dev(out, "out")
    dt = _dtype_code(dO)
    need = conv_bwd_data_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m)
    if need == 2**64 - 1:
        raise SdgpError(-3, "sdgp_conv_bwd_data_workspace")
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=dO.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().sdgp_conv_bwd_data(_ptr(dO), _ptr(W), _ptr(out), B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m,
                                   ranker, seed & (2**64 - 1), _ptr(workspace), wbytes, _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_conv_bwd_data")
    return out
