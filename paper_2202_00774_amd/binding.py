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
           "sdgp_conv_bwd_data_noalloc",
           "sdgp_channel_scales_workspace", "sdgp_channel_scales", "sdgp_prune_channel_rescaled", "sdgp_scale_filter",
           "sdgp_conv_bwd_data_channel_rescaled_workspace", "sdgp_conv_bwd_data_channel_rescaled",
           "sdgp_conv_bwd_data_compact_workspace", "sdgp_conv_bwd_data_compact",
           "sdgp_conv_bwd_data_grouped_workspace", "sdgp_conv_bwd_data_grouped",
           "sdgp_conv_fwd_workspace", "sdgp_conv_fwd", "sdgp_conv_bwd_weight_workspace", "sdgp_conv_bwd_weight",
           "sdgp_peak_probe", "sdgp_status_string", "sdgp_version")


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
            lib.sdgp_conv_bwd_data_noalloc.restype = i32
            lib.sdgp_conv_bwd_data_noalloc.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32,
                                                       i32, i32, u64, vp]
            lib.sdgp_conv_bwd_data_workspace.restype = sz
            lib.sdgp_conv_bwd_data_workspace.argtypes = [i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32, i32]
            lib.sdgp_channel_scales_workspace.restype = sz
            lib.sdgp_channel_scales_workspace.argtypes = [i64, i64, i32, i32, i32]
            lib.sdgp_channel_scales.restype = i32
            lib.sdgp_channel_scales.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, sz, vp]
            lib.sdgp_prune_channel_rescaled.restype = i32
            lib.sdgp_prune_channel_rescaled.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp]
            lib.sdgp_scale_filter.restype = i32
            lib.sdgp_scale_filter.argtypes = [vp, vp, vp, i64, i64, i32, vp]
            lib.sdgp_conv_bwd_data_channel_rescaled_workspace.restype = sz
            lib.sdgp_conv_bwd_data_channel_rescaled_workspace.argtypes = [i64, i64, i64, i64, i64, i32, i32, i32, i32,
                                                                         i32, i32, i32]
            lib.sdgp_conv_bwd_data_channel_rescaled.restype = i32
            lib.sdgp_conv_bwd_data_channel_rescaled.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32,
                                                               i32, i32, i32, vp, sz, vp]
            lib.sdgp_conv_bwd_data_compact_workspace.restype = sz
            lib.sdgp_conv_bwd_data_compact_workspace.argtypes = [i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32, i32]
            lib.sdgp_conv_bwd_data_grouped_workspace.restype = sz
            lib.sdgp_conv_bwd_data_grouped_workspace.argtypes = [i64, i64, i64, i64, i64, i32, i32, i32, i32, i64, i32, i32, i32]
            lib.sdgp_conv_bwd_data_grouped.restype = i32
            lib.sdgp_conv_bwd_data_grouped.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i64, i32, i32,
                                                       i32, i32, u64, vp, sz, vp]
            lib.sdgp_conv_bwd_data_compact.restype = i32
            lib.sdgp_conv_bwd_data_compact.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32, i32,
                                                       i32, u64, vp, sz, vp]
            geom = [i64, i64, i64, i64, i64, i32, i32, i32, i32, i32]
            lib.sdgp_conv_fwd_workspace.restype = sz
            lib.sdgp_conv_fwd_workspace.argtypes = geom
            lib.sdgp_conv_fwd.restype = i32
            lib.sdgp_conv_fwd.argtypes = [vp, vp, vp] + geom + [vp, sz, vp]
            lib.sdgp_conv_bwd_weight_workspace.restype = sz
            lib.sdgp_conv_bwd_weight_workspace.argtypes = geom
            lib.sdgp_conv_bwd_weight.restype = i32
            lib.sdgp_conv_bwd_weight.argtypes = [vp, vp, vp] + geom + [vp, sz, vp]
            lib.sdgp_peak_probe.restype = i32
            lib.sdgp_peak_probe.argtypes = [i32, vp, vp, sz, i32, ctypes.POINTER(ctypes.c_double), vp]
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


def sdgp_conv_bwd_data_noalloc(dO: torch.Tensor, W: torch.Tensor, H: int, Wd: int, stride: int, pad: int, n: int, m: int,
                               ranker: int, seed: int, out: torch.Tensor) -> torch.Tensor:
    """sdgp_conv_bwd_data into the caller's ``out`` without a workspace: scratch comes from the library's own array."""
    _dev(dO, "dO"), _dev(W, "W"), _dev(out, "out")
    if dO.dim() != 4 or W.dim() != 4 or W.shape[0] != dO.shape[3] or W.dtype != dO.dtype:
        raise ValueError("expected dO [B,P,Q,C_out] and W [C_out,R,S,C_in] of one dtype")
    B, P, Q, C_out = dO.shape
    _, R, S, C_in = W.shape
    if (H + 2 * pad - R) // stride + 1 != P or (Wd + 2 * pad - S) // stride + 1 != Q:
        raise ValueError("dO's spatial size does not match H, Wd, stride, pad")
    if tuple(out.shape) != (B, H, Wd, C_in) or out.dtype != dO.dtype:
        raise ValueError("out must be [B,H,Wd,C_in] of dO's dtype")
    rc = load().sdgp_conv_bwd_data_noalloc(_ptr(dO), _ptr(W), _ptr(out), B, H, Wd, C_in, C_out, R, S, stride, pad,
                                           _dtype_code(dO), n, m, ranker, seed & (2**64 - 1), _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_conv_bwd_data_noalloc")
    return out


# ---------------------------------------------- Rescaled Magnitude, one factor per channel

_INVALID = 2**64 - 1


def _workspace(need: int, workspace, device, where: str):
    if need == _INVALID:
        raise SdgpError(-3, where)
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def sdgp_channel_scales(dO: torch.Tensor, n: int, m: int, *, sums: bool = False, workspace: torch.Tensor | None = None):
    """Per-channel factors of ``dO`` ([..., C]) under Magnitude n:m pruning: fp32 [C]; with ``sums`` also the two
    fp64 column sums as a [2, C] tensor (all |x|, kept |x|)."""
    _dev(dO, "dO")
    C = dO.shape[-1]
    rows = dO.numel() // C if C else 0
    dt = _dtype_code(dO)
    lib = load()
    workspace, wbytes = _workspace(int(lib.sdgp_channel_scales_workspace(rows, C, dt, n, m)), workspace, dO.device,
                                   "sdgp_channel_scales_workspace")
    scale = torch.empty(C, dtype=torch.float32, device=dO.device)
    both = torch.empty((2, C), dtype=torch.float64, device=dO.device) if sums else None
    rc = lib.sdgp_channel_scales(_ptr(dO), rows, C, dt, n, m, _ptr(scale), _ptr(both), _ptr(workspace), wbytes, _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_channel_scales")
    return (scale, both) if sums else scale


def sdgp_prune_channel_rescaled(dO: torch.Tensor, n: int, m: int, scale: torch.Tensor | None = None) -> torch.Tensor:
    """Magnitude n:m pruning of ``dO`` with kept values multiplied by their channel's factor (computed when not given)."""
    _dev(dO, "dO")
    C = dO.shape[-1]
    rows = dO.numel() // C if C else 0
    if scale is None:
        scale = sdgp_channel_scales(dO, n, m)
    _dev(scale, "scale")
    if scale.dtype != torch.float32 or scale.numel() != C:
        raise ValueError("scale must be float32 [C]")
    out = torch.empty_like(dO)
    rc = load().sdgp_prune_channel_rescaled(_ptr(dO), rows, C, _dtype_code(dO), n, m, _ptr(scale), _ptr(out), _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_prune_channel_rescaled")
    return out


def sdgp_scale_filter(W: torch.Tensor, scale: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """``W[k, ...] * scale[k]`` for a filter whose first axis is C_out."""
    _dev(W, "W"), _dev(scale, "scale")
    C_out = W.shape[0]
    if scale.dtype != torch.float32 or scale.numel() != C_out:
        raise ValueError("scale must be float32 [C_out]")
    if out is None:
        out = torch.empty_like(W)
    _dev(out, "out")
    inner = W.numel() // C_out if C_out else 0
    rc = load().sdgp_scale_filter(_ptr(W), _ptr(scale), _ptr(out), C_out, inner, _dtype_code(W), _stream(W))
    if rc != 0:
        raise SdgpError(rc, "sdgp_scale_filter")
    return out


def sdgp_peak_probe(kind: int, a: torch.Tensor | None, b: torch.Tensor, nbytes: int = 0, iters: int = 1) -> float:
    """One launch of a measurement kernel (0 copy a -> b, 1 read a, 2 dense / 3 structured-sparse matrix instructions);
    returns the bytes or floating-point operations of the launch.  The caller times it."""
    _dev(b, "b")
    if a is not None:
        _dev(a, "a")
    work = ctypes.c_double(0.0)
    rc = load().sdgp_peak_probe(int(kind), _ptr(a) if a is not None else None, _ptr(b), int(nbytes), int(iters),
                                ctypes.byref(work), _stream(b))
    if rc != 0:
        raise SdgpError(rc, "sdgp_peak_probe")
    return work.value


def sdgp_conv_bwd_data_channel_rescaled(dO: torch.Tensor, W: torch.Tensor, H: int, Wd: int, stride: int, pad: int,
                                        n: int, m: int, out: torch.Tensor | None = None,
                                        workspace: torch.Tensor | None = None) -> torch.Tensor:
    """dD of a convolution from dO pruned by Magnitude and rescaled per channel, in one call."""
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
    lib = load()
    need = int(lib.sdgp_conv_bwd_data_channel_rescaled_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m))
    workspace, wbytes = _workspace(need, workspace, dO.device, "sdgp_conv_bwd_data_channel_rescaled_workspace")
    rc = lib.sdgp_conv_bwd_data_channel_rescaled(_ptr(dO), _ptr(W), _ptr(out), B, H, Wd, C_in, C_out, R, S, stride, pad,
                                                 dt, n, m, _ptr(workspace), wbytes, _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_conv_bwd_data_channel_rescaled")
    return out


def sdgp_linear_bwd_data_channel_rescaled(dO: torch.Tensor, W: torch.Tensor, n: int, m: int) -> torch.Tensor:
    """The same for a linear layer (dO [rows, C_out], W [C_out, C_in]): a 1x1 convolution over rows pixels."""
    if dO.dim() != 2 or W.dim() != 2:
        raise ValueError("expected dO [rows, C_out] and W [C_out, C_in]")
    rows, C_out = dO.shape
    out = sdgp_conv_bwd_data_channel_rescaled(dO.view(rows, 1, 1, C_out), W.view(C_out, 1, 1, W.shape[1]), 1, 1, 1, 0, n, m)
    return out.view(rows, W.shape[1])


def sdgp_conv_bwd_data_compact(dO: torch.Tensor, W: torch.Tensor, H: int, Wd: int, stride: int, pad: int, n: int, m: int,
                               ranker: int, seed: int = 0, out: torch.Tensor | None = None,
                               workspace: torch.Tensor | None = None) -> torch.Tensor:
    """sdgp_conv_bwd_data through the compacted gradient: prune pass to (values, positions), then one AXPY per kept value."""
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
    lib = load()
    need = int(lib.sdgp_conv_bwd_data_compact_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m))
    workspace, wbytes = _workspace(need, workspace, dO.device, "sdgp_conv_bwd_data_compact_workspace")
    rc = lib.sdgp_conv_bwd_data_compact(_ptr(dO), _ptr(W), _ptr(out), B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m,
                                        ranker, seed & (2**64 - 1), _ptr(workspace), wbytes, _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_conv_bwd_data_compact")
    return out


def sdgp_conv_bwd_data_grouped(dO: torch.Tensor, W: torch.Tensor, H: int, Wd: int, stride: int, pad: int, groups: int,
                               n: int, m: int, ranker: int, seed: int = 0, out: torch.Tensor | None = None,
                               workspace: torch.Tensor | None = None) -> torch.Tensor:
    """sdgp_conv_bwd_data for a grouped convolution: dO [B,P,Q,C_out], W [C_out,R,S,C_in/groups] -> dD [B,H,Wd,C_in]."""
    _dev(dO, "dO"), _dev(W, "W")
    if dO.dim() != 4 or W.dim() != 4 or W.shape[0] != dO.shape[3] or W.dtype != dO.dtype:
        raise ValueError("expected dO [B,P,Q,C_out] and W [C_out,R,S,C_in/groups] of one dtype")
    B, P, Q, C_out = dO.shape
    _, R, S, cig = W.shape
    C_in = cig * groups
    if (H + 2 * pad - R) // stride + 1 != P or (Wd + 2 * pad - S) // stride + 1 != Q:
        raise ValueError("dO's spatial size does not match H, Wd, stride, pad")
    if out is None:
        out = torch.empty((B, H, Wd, C_in), dtype=dO.dtype, device=dO.device)
    _dev(out, "out")
    dt = _dtype_code(dO)
    lib = load()
    need = int(lib.sdgp_conv_bwd_data_grouped_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt, n, m))
    workspace, wbytes = _workspace(need, workspace, dO.device, "sdgp_conv_bwd_data_grouped_workspace")
    rc = lib.sdgp_conv_bwd_data_grouped(_ptr(dO), _ptr(W), _ptr(out), B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt,
                                        n, m, ranker, seed & (2**64 - 1), _ptr(workspace), wbytes, _stream(dO))
    if rc != 0:
        raise SdgpError(rc, "sdgp_conv_bwd_data_grouped")
    return out


# ---------------------------------------------- the two other products of a layer's step (nothing is pruned)

def sdgp_conv_fwd(D: torch.Tensor, W: torch.Tensor, stride: int, pad: int, out: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None) -> torch.Tensor:
    """O [B,P,Q,C_out] from D [B,H,Wd,C_in] (NHWC) and W [C_out,R,S,C_in]."""
    _dev(D, "D"), _dev(W, "W")
    if D.dim() != 4 or W.dim() != 4 or W.shape[3] != D.shape[3] or W.dtype != D.dtype:
        raise ValueError("expected D [B,H,Wd,C_in] and W [C_out,R,S,C_in] of one dtype")
    B, H, Wd, C_in = D.shape
    C_out, R, S, _ = W.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    if out is None:
        out = torch.empty((B, max(P, 0), max(Q, 0), C_out), dtype=D.dtype, device=D.device)
    _dev(out, "out")
    dt = _dtype_code(D)
    lib = load()
    need = int(lib.sdgp_conv_fwd_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt))
    workspace, wbytes = _workspace(need, workspace, D.device, "sdgp_conv_fwd_workspace")
    rc = lib.sdgp_conv_fwd(_ptr(D), _ptr(W), _ptr(out), B, H, Wd, C_in, C_out, R, S, stride, pad, dt, _ptr(workspace), wbytes,
                           _stream(D))
    if rc != 0:
        raise SdgpError(rc, "sdgp_conv_fwd")
    return out


def sdgp_conv_bwd_weight(D: torch.Tensor, dO: torch.Tensor, R: int, S: int, stride: int, pad: int,
                         out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """dW [C_out,R,S,C_in] in float32 from D [B,H,Wd,C_in] and the unpruned dO [B,P,Q,C_out]."""
    _dev(D, "D"), _dev(dO, "dO")
    if D.dim() != 4 or dO.dim() != 4 or dO.shape[0] != D.shape[0] or dO.dtype != D.dtype:
        raise ValueError("expected D [B,H,Wd,C_in] and dO [B,P,Q,C_out] of one dtype")
    B, H, Wd, C_in = D.shape
    _, P, Q, C_out = dO.shape
    if (H + 2 * pad - R) // stride + 1 != P or (Wd + 2 * pad - S) // stride + 1 != Q:
        raise ValueError("dO's spatial size does not match D, R, S, stride, pad")
    if out is None:
        out = torch.empty((C_out, R, S, C_in), dtype=torch.float32, device=D.device)
    _dev(out, "out")
    if out.dtype != torch.float32 or tuple(out.shape) != (C_out, R, S, C_in):
        raise ValueError("out must be float32 [C_out,R,S,C_in]")
    dt = _dtype_code(D)
    lib = load()
    need = int(lib.sdgp_conv_bwd_weight_workspace(B, H, Wd, C_in, C_out, R, S, stride, pad, dt))
    workspace, wbytes = _workspace(need, workspace, D.device, "sdgp_conv_bwd_weight_workspace")
    rc = lib.sdgp_conv_bwd_weight(_ptr(D), _ptr(dO), _ptr(out), B, H, Wd, C_in, C_out, R, S, stride, pad, dt,
                                  _ptr(workspace), wbytes, _stream(D))
    if rc != 0:
        raise SdgpError(rc, "sdgp_conv_bwd_weight")
    return out
