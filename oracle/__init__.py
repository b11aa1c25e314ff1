"""CPU oracle of the SDGP backward-data path -- TEST INFRASTRUCTURE ONLY.

A thin ctypes front of ``sdgp_oracle.c`` (plain C, host memory, fp64
accumulation).  Only the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library and its Python
binding never do, and the two share no code.

All arrays are numpy arrays in host memory.  bfloat16 tensors travel as
``uint16`` bit patterns, fp32 tensors as ``float32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

F32, BF16 = 0, 1
RANDOM, GREEDY, GREEDY_ADJUSTED = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdgp_oracle.c")
_LIB = os.path.join(_HERE, "libsdgp_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: no fast-math, no FMA contraction, OpenMP over rows."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB + ".tmp", _SRC]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i64, u64, i32, vp = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p
            lib.sdgp_ref_hash.restype = ctypes.c_uint32
            lib.sdgp_ref_hash.argtypes = [u64, u64]
            lib.sdgp_ref_float_to_bf16.restype = ctypes.c_uint16
            lib.sdgp_ref_float_to_bf16.argtypes = [ctypes.c_float]
            lib.sdgp_ref_bf16_to_float.restype = ctypes.c_float
            lib.sdgp_ref_bf16_to_float.argtypes = [ctypes.c_uint16]
            lib.sdgp_ref_prune.restype = i32
            lib.sdgp_ref_prune.argtypes = [vp, i64, i64, i32, i32, i32, i32, u64, vp, vp, vp]
            lib.sdgp_ref_prune_channel_rescaled.restype = i32
            lib.sdgp_ref_prune_channel_rescaled.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
            lib.sdgp_ref_linear_bwd_data.restype = i32
            lib.sdgp_ref_linear_bwd_data.argtypes = [vp, vp, i64, i64, i64, i32, vp, vp]
            lib.sdgp_ref_conv_bwd_data.restype = i32
            lib.sdgp_ref_conv_bwd_data.argtypes = [vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32,
                                                   i32, vp, vp]
            lib.sdgp_ref_conv_bwd_data_at.restype = i32
            lib.sdgp_ref_conv_bwd_data_at.argtypes = [vp, vp, i64, i64, i64, i64, i64, i32, i32, i32,
                                                      i32, i32, vp, i64, vp, vp]
            lib.sdgp_ref_conv_fwd.restype = i32
            lib.sdgp_ref_conv_fwd.argtypes = [vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, vp, i64, vp, vp]
            lib.sdgp_ref_conv_bwd_weight.restype = i32
            lib.sdgp_ref_conv_bwd_weight.argtypes = [vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, vp, i64,
                                                     vp, vp]
            lib.sdgp_ref_conv_bwd_data_grouped.restype = i32
            lib.sdgp_ref_conv_bwd_data_grouped.argtypes = [vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i64, i32, vp, i64,
                                                           vp, vp]
            lib.sdgp_ref_threads.restype = i32
            lib.sdgp_ref_threads.argtypes = []
            _lib = lib
    return _lib


def _np_dtype(dtype: int):
    if dtype == F32:
        return np.float32
    if dtype == BF16:
        return np.uint16
    raise ValueError("dtype must be F32 or BF16")


def _check(a: np.ndarray, dtype: int, name: str) -> np.ndarray:
    if a.dtype != _np_dtype(dtype):
        raise TypeError(f"{name}: expected {_np_dtype(dtype).__name__} storage, got {a.dtype}")
    return np.ascontiguousarray(a)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().sdgp_ref_threads())


def hash32(seed: int, e: int) -> int:
    """Key of flat element ``e`` under ``seed`` for the random ranker."""
    return int(_load().sdgp_ref_hash(seed & (2**64 - 1), e & (2**64 - 1)))


def float_to_bf16(x: float) -> int:
    return int(_load().sdgp_ref_float_to_bf16(float(x)))


def bf16_to_float(h: int) -> float:
    return float(_load().sdgp_ref_bf16_to_float(int(h)))


def prune(dO: np.ndarray, n: int, m: int, ranker: int, seed: int = 0, dtype: int | None = None):
    """Alg. 1 on ``dO`` viewed as [rows, C] (C = last axis).

    Returns ``(pruned, vals, idx)``: the dense-shaped pruned copy, the kept
    values [rows, C*n/m] and their in-group positions (uint8).
    """
    if dtype is None:
        dtype = F32 if dO.dtype == np.float32 else BF16
    dO = _check(dO, dtype, "dO")
    C = dO.shape[-1]
    rows = dO.size // C if C else 0
    if m < 1 or C % m:
        raise ValueError("C must be a multiple of m")
    pruned = np.empty_like(dO)
    vals = np.empty(dO.shape[:-1] + (C // m * n,), dO.dtype)
    idx = np.empty(dO.shape[:-1] + (C // m * n,), np.uint8)
    rc = _load().sdgp_ref_prune(_ptr(dO), rows, C, dtype, n, m, ranker, seed & (2**64 - 1),
                                _ptr(pruned), _ptr(vals), _ptr(idx))
    if rc != 0:
        raise ValueError("sdgp_ref_prune rejected its arguments")
    return pruned, vals, idx


def prune_channel_rescaled(dO: np.ndarray, n: int, m: int, dtype: int | None = None):
    """Magnitude pruning with one rescaling factor per channel (second reading of Rescaled Magnitude).

    ``dO`` is viewed as [rows, C].  Returns ``(pruned, scale, total, kept)``: the dense-shaped pruned copy,
    the fp32 factor of every channel and the two fp64 column sums it is the quotient of.
    """
    if dtype is None:
        dtype = F32 if dO.dtype == np.float32 else BF16
    dO = _check(dO, dtype, "dO")
    C = dO.shape[-1]
    rows = dO.size // C if C else 0
    if m < 1 or C % m:
        raise ValueError("C must be a multiple of m")
    pruned = np.empty_like(dO)
    scale = np.empty(C, np.float32)
    total = np.empty(C, np.float64)
    kept = np.empty(C, np.float64)
    rc = _load().sdgp_ref_prune_channel_rescaled(_ptr(dO), rows, C, dtype, n, m, _ptr(total), _ptr(kept),
                                                 _ptr(scale), _ptr(pruned))
    if rc != 0:
        raise ValueError("sdgp_ref_prune_channel_rescaled rejected its arguments")
    return pruned, scale, total, kept


def linear_bwd_data(dOp: np.ndarray, W: np.ndarray, dtype: int | None = None):
    """dD = dOp @ W in fp64 for the already pruned dOp [rows, C_out], W [C_out, C_in].

    Returns ``(dD, absum)`` with ``absum = |dOp| @ |W|``.
    """
    if dtype is None:
        dtype = F32 if dOp.dtype == np.float32 else BF16
    dOp, W = _check(dOp, dtype, "dOp"), _check(W, dtype, "W")
    rows, C_out = dOp.shape
    if W.shape[0] != C_out:
        raise ValueError("W must be [C_out, C_in]")
    C_in = W.shape[1]
    dD = np.empty((rows, C_in), np.float64)
    ab = np.empty((rows, C_in), np.float64)
    rc = _load().sdgp_ref_linear_bwd_data(_ptr(dOp), _ptr(W), rows, C_out, C_in, dtype, _ptr(dD), _ptr(ab))
    if rc != 0:
        raise ValueError("sdgp_ref_linear_bwd_data rejected its arguments")
    return dD, ab


def conv_out_size(H: int, R: int, stride: int, pad: int) -> int:
    return (H + 2 * pad - R) // stride + 1


def conv_bwd_data(dOp: np.ndarray, W: np.ndarray, H: int, Wd: int, stride: int, pad: int,
                  dtype: int | None = None, pixels: np.ndarray | None = None):
    """Backward-data of a convolution for the already pruned dOp [B,P,Q,C_out], W [C_out,R,S,C_in].

    Returns ``(dD, absum)`` as fp64 [B,H,Wd,C_in]; with ``pixels`` (flat
    ``(b*H+h)*Wd+w`` indices) only those input pixels, as [len(pixels), C_in].
    """
    if dtype is None:
        dtype = F32 if dOp.dtype == np.float32 else BF16
    dOp, W = _check(dOp, dtype, "dOp"), _check(W, dtype, "W")
    B, P, Q, C_out = dOp.shape
    K, R, S, C_in = W.shape
    if K != C_out:
        raise ValueError("W must be [C_out, R, S, C_in]")
    if P != conv_out_size(H, R, stride, pad) or Q != conv_out_size(Wd, S, stride, pad):
        raise ValueError("dOp spatial size does not match H, Wd, stride, pad")
    lib = _load()
    if pixels is None:
        dD = np.empty((B, H, Wd, C_in), np.float64)
        ab = np.empty((B, H, Wd, C_in), np.float64)
        rc = lib.sdgp_ref_conv_bwd_data(_ptr(dOp), _ptr(W), B, H, Wd, C_in, C_out, R, S, stride, pad,
                                        dtype, _ptr(dD), _ptr(ab))
    else:
        pixels = np.ascontiguousarray(pixels, dtype=np.int64)
        dD = np.empty((pixels.size, C_in), np.float64)
        ab = np.empty((pixels.size, C_in), np.float64)
        rc = lib.sdgp_ref_conv_bwd_data_at(_ptr(dOp), _ptr(W), B, H, Wd, C_in, C_out, R, S, stride, pad,
                                           dtype, _ptr(pixels), pixels.size, _ptr(dD), _ptr(ab))
    if rc != 0:
        raise ValueError("sdgp_ref_conv_bwd_data rejected its arguments")
    return dD, ab


def conv_bwd_data_grouped(dOp: np.ndarray, W: np.ndarray, H: int, Wd: int, stride: int, pad: int, groups: int,
                          dtype: int | None = None, pixels: np.ndarray | None = None):
    """Backward-data of a grouped convolution (the RegNetX layers of Sec. IV) for the already pruned dOp
    [B,P,Q,C_out] and W [C_out,R,S,C_in/groups].

    Returns ``(dD, absum)`` as fp64 [B,H,Wd,C_in]; with ``pixels`` (flat ``(b*H+h)*Wd+w`` indices) only those input
    pixels, as [len(pixels), C_in].
    """
    if dtype is None:
        dtype = F32 if dOp.dtype == np.float32 else BF16
    dOp, W = _check(dOp, dtype, "dOp"), _check(W, dtype, "W")
    B, P, Q, C_out = dOp.shape
    K, R, S, cig = W.shape
    if K != C_out:
        raise ValueError("W must be [C_out, R, S, C_in/groups]")
    if P != conv_out_size(H, R, stride, pad) or Q != conv_out_size(Wd, S, stride, pad):
        raise ValueError("dOp spatial size does not match H, Wd, stride, pad")
    C_in = cig * groups
    lib = _load()
    if pixels is None:
        shape, pp, count = (B, H, Wd, C_in), None, 0
    else:
        pixels = np.ascontiguousarray(pixels, dtype=np.int64)
        shape, pp, count = (pixels.size, C_in), _ptr(pixels), pixels.size
    dD, ab = np.empty(shape, np.float64), np.empty(shape, np.float64)
    rc = lib.sdgp_ref_conv_bwd_data_grouped(_ptr(dOp), _ptr(W), B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dtype,
                                            pp, count, _ptr(dD), _ptr(ab))
    if rc != 0:
        raise ValueError("sdgp_ref_conv_bwd_data_grouped rejected its arguments")
    return dD, ab


def conv_fwd(D: np.ndarray, W: np.ndarray, stride: int, pad: int, dtype: int | None = None,
             pixels: np.ndarray | None = None):
    """Forward convolution of D [B,H,Wd,C_in] with W [C_out,R,S,C_in] (Sec. II-A, Fig. 1).

    Returns ``(O, absum)`` as fp64 [B,P,Q,C_out]; with ``pixels`` (flat ``(b*P+p)*Q+q`` indices) only those output
    pixels, as [len(pixels), C_out].
    """
    if dtype is None:
        dtype = F32 if D.dtype == np.float32 else BF16
    D, W = _check(D, dtype, "D"), _check(W, dtype, "W")
    B, H, Wd, C_in = D.shape
    C_out, R, S, C2 = W.shape
    if C2 != C_in:
        raise ValueError("W must be [C_out, R, S, C_in]")
    P, Q = conv_out_size(H, R, stride, pad), conv_out_size(Wd, S, stride, pad)
    if pixels is None:
        shape, px, cnt = (B, P, Q, C_out), None, 0
    else:
        px = np.ascontiguousarray(pixels, dtype=np.int64)
        shape, cnt = (px.size, C_out), px.size
    O, ab = np.empty(shape, np.float64), np.empty(shape, np.float64)
    rc = _load().sdgp_ref_conv_fwd(_ptr(D), _ptr(W), B, H, Wd, C_in, C_out, R, S, stride, pad, dtype, _ptr(px), cnt,
                                   _ptr(O), _ptr(ab))
    if rc != 0:
        raise ValueError("sdgp_ref_conv_fwd rejected its arguments")
    return O, ab


def conv_bwd_weight(D: np.ndarray, dO: np.ndarray, R: int, S: int, stride: int, pad: int, dtype: int | None = None,
                    entries: np.ndarray | None = None):
    """Weight gradient from D [B,H,Wd,C_in] and the UNPRUNED dO [B,P,Q,C_out] (Sec. II-A, Fig. 1; Sec. III-A).

    Returns ``(dW, absum)`` as fp64 [C_out,R,S,C_in]; with ``entries`` (flat ``((k*R+r)*S+s)*C_in+c`` indices) only
    those filter elements, as [len(entries)].
    """
    if dtype is None:
        dtype = F32 if D.dtype == np.float32 else BF16
    D, dO = _check(D, dtype, "D"), _check(dO, dtype, "dO")
    B, H, Wd, C_in = D.shape
    B2, P, Q, C_out = dO.shape
    if B2 != B or P != conv_out_size(H, R, stride, pad) or Q != conv_out_size(Wd, S, stride, pad):
        raise ValueError("dO does not match D, R, S, stride, pad")
    if entries is None:
        shape, en, cnt = (C_out, R, S, C_in), None, 0
    else:
        en = np.ascontiguousarray(entries, dtype=np.int64)
        shape, cnt = (en.size,), en.size
    dW, ab = np.empty(shape, np.float64), np.empty(shape, np.float64)
    rc = _load().sdgp_ref_conv_bwd_weight(_ptr(D), _ptr(dO), B, H, Wd, C_in, C_out, R, S, stride, pad, dtype, _ptr(en),
                                          cnt, _ptr(dW), _ptr(ab))
    if rc != 0:
        raise ValueError("sdgp_ref_conv_bwd_weight rejected its arguments")
    return dW, ab
