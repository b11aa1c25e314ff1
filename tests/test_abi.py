"""The C ABI without a GPU: the library loads, exports what include/sdgp.h declares, and validates arguments
before touching the device (so every error path can be driven from a CPU-only machine)."""
import ctypes
import os
import re

import pytest

from paper_2202_00774_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, E_NULL, E_NM, E_SHAPE, E_DTYPE, E_RANKER, E_WS, E_HIP = 0, -1, -2, -3, -4, -5, -6, -7
P = ctypes.c_void_p(16)       # never dereferenced: validation fails first


@pytest.fixture(scope="module")
def lib():
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sdgp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sdgp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_function(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    seen = set()
    for code in range(0, -8, -1):
        s = binding.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert binding.status_string(-99) == "unknown status"
    assert binding.version() >= 100


def prune(lib, rows=4, C=16, dt=1, n=2, m=4, rk=1, dO=P, pruned=P, vals=None, idx=None):
    return lib.sdgp_prune(dO, rows, C, dt, n, m, rk, 0, pruned, vals, idx, None)


def test_prune_argument_errors(lib):
    assert prune(lib, dt=2) == E_DTYPE
    assert prune(lib, rk=3) == E_RANKER
    assert prune(lib, rk=-1) == E_RANKER
    for n, m in ((0, 4), (5, 4), (2, 33), (-1, 4)):
        assert prune(lib, n=n, m=m, C=m * 4 if m > 0 else 16) == E_NM
    assert prune(lib, C=18) == E_SHAPE                 # 18 % 4 != 0
    assert prune(lib, rows=-1) == E_SHAPE
    assert prune(lib, rows=2 ** 40, C=2 ** 30) == E_SHAPE
    assert prune(lib, dO=None) == E_NULL
    assert prune(lib, pruned=None) == E_NULL           # no output requested
    assert prune(lib, vals=P, idx=None) == E_NULL      # vals without idx
    assert prune(lib, vals=None, idx=P) == E_NULL
    assert prune(lib, rows=0) == OK                    # empty tensor: nothing to do
    assert prune(lib, rows=0, dO=None) == OK
    assert prune(lib, C=0) == OK


def linear(lib, rows=4, C_out=16, C_in=8, dt=1, n=2, m=4, rk=1, dO=P, W=P, dD=P):
    return lib.sdgp_linear_bwd_data(dO, W, dD, rows, C_out, C_in, dt, n, m, rk, 0, None)


def test_linear_argument_errors(lib):
    assert linear(lib, dt=7) == E_DTYPE
    assert linear(lib, rk=9) == E_RANKER
    assert linear(lib, n=3, m=2) == E_NM
    assert linear(lib, C_out=18) == E_SHAPE
    assert linear(lib, rows=-2) == E_SHAPE
    assert linear(lib, C_in=-1) == E_SHAPE
    assert linear(lib, dO=None) == E_NULL
    assert linear(lib, W=None) == E_NULL
    assert linear(lib, dD=None) == E_NULL
    assert linear(lib, rows=0) == OK
    assert linear(lib, C_in=0) == OK


def conv(lib, B=2, H=8, Wd=8, C_in=8, C_out=16, R=3, S=3, stride=1, pad=1, dt=1, n=2, m=4, rk=1, dO=P, W=P, dD=P,
         ws=None, ws_bytes=0):
    return lib.sdgp_conv_bwd_data(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, 0, ws, ws_bytes, None)


def test_conv_argument_errors(lib):
    assert conv(lib, dt=-1) == E_DTYPE
    assert conv(lib, rk=5) == E_RANKER
    assert conv(lib, n=0) == E_NM
    assert conv(lib, C_out=10) == E_SHAPE
    assert conv(lib, R=0) == E_SHAPE
    assert conv(lib, S=12) == E_SHAPE
    assert conv(lib, stride=0) == E_SHAPE
    assert conv(lib, stride=5) == E_SHAPE
    assert conv(lib, pad=3) == E_SHAPE                  # pad >= R
    assert conv(lib, pad=-1) == E_SHAPE
    assert conv(lib, H=1, Wd=1, R=5, S=5, pad=1) == E_SHAPE   # filter larger than the padded input
    assert conv(lib, B=-1) == E_SHAPE
    assert conv(lib, dO=None) == E_NULL
    assert conv(lib, W=None) == E_NULL
    assert conv(lib, dD=None) == E_NULL
    assert conv(lib, B=0) == OK
    assert conv(lib, C_in=0) == OK
    bad = ctypes.c_size_t(-1).value
    assert lib.sdgp_conv_bwd_data_workspace(2, 8, 8, 8, 10, 3, 3, 1, 1, 1, 2, 4) == bad
    assert lib.sdgp_conv_bwd_data_workspace(2, 8, 8, 8, 16, 3, 3, 1, 1, 1, 2, 4) != bad


def test_first_layer_workspace_query(lib):
    # 7x7 stride 2 pad 3 on an even image: 16 window positions x 16 columns of 80 bytes per 32 output channels
    assert lib.sdgp_conv_bwd_data_workspace(256, 224, 224, 3, 64, 7, 7, 2, 3, 1, 2, 4) == 2 * 20 * 1024
    assert lib.sdgp_conv_bwd_data_workspace(256, 224, 224, 3, 128, 7, 7, 2, 3, 1, 4, 4) == 4 * 20 * 1024
    # other 7x7 layers on three channels (here: an odd image): 160 (tap, channel) columns of 144 bytes, in whole KB,
    # per 64 output channels
    assert lib.sdgp_conv_bwd_data_workspace(4, 223, 223, 3, 64, 7, 7, 2, 3, 1, 2, 4) == 23 * 1024
    assert lib.sdgp_conv_bwd_data_workspace(4, 223, 223, 3, 128, 7, 7, 2, 3, 1, 4, 4) == 2 * 23 * 1024
    # 3x3 on three channels fits one column tile: no image; fp32 and wide layers never ask
    assert lib.sdgp_conv_bwd_data_workspace(512, 32, 32, 3, 64, 3, 3, 1, 1, 1, 2, 4) == 0
    assert lib.sdgp_conv_bwd_data_workspace(256, 224, 224, 3, 64, 7, 7, 2, 3, 0, 2, 4) == 0
    assert lib.sdgp_conv_bwd_data_workspace(512, 32, 32, 64, 128, 3, 3, 1, 1, 1, 2, 4) == 0


def test_workspace_too_small_is_rejected(lib):
    # wherever the library asks for workspace, passing none or too little is an error before any launch
    shapes = [(512, 32, 32, 64, 128, 3, 3, 1, 1), (128, 56, 56, 256, 64, 1, 1, 1, 0), (256, 56, 56, 128, 128, 3, 3, 2, 1),
              (256, 224, 224, 3, 64, 7, 7, 2, 3), (512, 32, 32, 3, 64, 3, 3, 1, 1)]   # first layers: the 7x7 one wants a filter image
    for B, H, Wd, C_in, C_out, R, S, st, pad in shapes:
        for n, m in ((2, 4), (2, 8), (4, 4)):
            need = lib.sdgp_conv_bwd_data_workspace(B, H, Wd, C_in, C_out, R, S, st, pad, 1, n, m)
            if need:
                assert conv(lib, B, H, Wd, C_in, C_out, R, S, st, pad, n=n, m=m) == E_WS
                assert conv(lib, B, H, Wd, C_in, C_out, R, S, st, pad, n=n, m=m, ws=P, ws_bytes=need - 1) == E_WS
                assert conv(lib, B, H, Wd, C_in, C_out, R, S, st, pad, n=n, m=m, ws=ctypes.c_void_p(8), ws_bytes=need) == E_WS


def test_noalloc_argument_errors(lib):
    """The entry point without a workspace: the checks of sdgp_conv_bwd_data, and a clear refusal when the problem
    wants more scratch than the library's own array holds (nothing is launched on these paths)."""
    def call(B=2, H=8, Wd=8, C_in=8, C_out=16, R=3, S=3, stride=1, pad=1, dt=1, n=2, m=4, rk=1, dO=P, W=P, dD=P):
        return lib.sdgp_conv_bwd_data_noalloc(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m, rk, 0, None)
    assert call(dt=-1) == E_DTYPE
    assert call(rk=5) == E_RANKER
    assert call(n=0) == E_NM
    assert call(C_out=10) == E_SHAPE
    assert call(dO=None) == E_NULL
    assert call(dD=None) == E_NULL
    assert call(B=0) == OK
    # the 7x7 stride-2 first layer wants 20 KB per 32 output channels: 384 channels fit the 256 KB array, 768 do not
    limit = 256 * 1024
    assert lib.sdgp_conv_bwd_data_workspace(2, 64, 64, 3, 384, 7, 7, 2, 3, 1, 2, 4) <= limit
    assert lib.sdgp_conv_bwd_data_workspace(2, 64, 64, 3, 768, 7, 7, 2, 3, 1, 2, 4) > limit
    assert call(B=2, H=64, Wd=64, C_in=3, C_out=768, R=7, S=7, stride=2, pad=3) == E_WS


# ------------------------------------------------ per-channel Rescaled Magnitude entry points

BAD = ctypes.c_size_t(-1).value


def test_channel_scales_argument_errors(lib):
    def scales(rows=4, C=16, dt=1, n=2, m=4, dO=P, scale=P, ws=P, ws_bytes=1 << 20):
        return lib.sdgp_channel_scales(dO, rows, C, dt, n, m, scale, None, ws, ws_bytes, None)

    assert scales(dt=3) == E_DTYPE
    assert scales(n=0) == E_NM
    assert scales(m=33, C=66) == E_NM
    assert scales(C=18) == E_SHAPE
    assert scales(rows=-1) == E_SHAPE
    assert scales(dO=None) == E_NULL
    assert scales(scale=None) == E_NULL
    assert scales(ws=None) == E_WS
    assert scales(ws_bytes=8) == E_WS
    assert scales(ws=ctypes.c_void_p(20)) == E_WS          # not 8-byte aligned
    assert scales(C=0) == OK
    assert lib.sdgp_channel_scales_workspace(4, 18, 1, 2, 4) == BAD
    need = lib.sdgp_channel_scales_workspace(1 << 20, 256, 1, 2, 4)
    assert need != BAD and need % 8 == 0 and 2 * 256 * 8 <= need <= (1 << 20) * 256 * 2 // 4   # far below the tensor
    assert lib.sdgp_channel_scales_workspace(4, 0, 1, 2, 4) == 0


def test_prune_channel_rescaled_and_scale_filter_argument_errors(lib):
    def prune_cr(rows=4, C=16, dt=1, n=2, m=4, dO=P, scale=P, pruned=P):
        return lib.sdgp_prune_channel_rescaled(dO, rows, C, dt, n, m, scale, pruned, None)

    assert prune_cr(dt=2) == E_DTYPE
    assert prune_cr(n=5) == E_NM
    assert prune_cr(C=6) == E_SHAPE
    assert prune_cr(dO=None) == E_NULL
    assert prune_cr(scale=None) == E_NULL
    assert prune_cr(pruned=None) == E_NULL
    assert prune_cr(rows=0) == OK

    def scale_filter(C_out=16, inner=72, dt=1, W=P, scale=P, out=P):
        return lib.sdgp_scale_filter(W, scale, out, C_out, inner, dt, None)

    assert scale_filter(dt=5) == E_DTYPE
    assert scale_filter(C_out=-1) == E_SHAPE
    assert scale_filter(inner=-1) == E_SHAPE
    assert scale_filter(W=None) == E_NULL
    assert scale_filter(scale=None) == E_NULL
    assert scale_filter(out=None) == E_NULL
    assert scale_filter(C_out=0) == OK
    assert scale_filter(inner=0) == OK


def test_conv_channel_rescaled_argument_errors(lib):
    def conv_cr(B=2, H=8, Wd=8, C_in=8, C_out=16, R=3, S=3, stride=1, pad=1, dt=1, n=2, m=4, dO=P, W=P, dD=P, ws=P,
                ws_bytes=1 << 24):
        return lib.sdgp_conv_bwd_data_channel_rescaled(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, dt, n, m,
                                                       ws, ws_bytes, None)

    assert conv_cr(dt=-1) == E_DTYPE
    assert conv_cr(n=0) == E_NM
    assert conv_cr(C_out=10) == E_SHAPE
    assert conv_cr(stride=5) == E_SHAPE
    assert conv_cr(dO=None) == E_NULL
    assert conv_cr(W=None) == E_NULL
    assert conv_cr(dD=None) == E_NULL
    assert conv_cr(ws=None) == E_WS
    need = lib.sdgp_conv_bwd_data_channel_rescaled_workspace(2, 8, 8, 8, 16, 3, 3, 1, 1, 1, 2, 4)
    assert need != BAD and need >= 16 * 4 + 16 * 9 * 8 * 2        # the factors and the rescaled filter at least
    assert conv_cr(ws_bytes=need - 1) == E_WS
    assert conv_cr(ws=ctypes.c_void_p(24)) == E_WS                # not 16-byte aligned
    assert conv_cr(B=0) == OK
    assert lib.sdgp_conv_bwd_data_channel_rescaled_workspace(2, 8, 8, 8, 10, 3, 3, 1, 1, 1, 2, 4) == BAD


def test_grouped_argument_errors(lib):
    def call(groups, C_in=32, C_out=64, n=2, m=4, dt=1, rk=1, dO=P, W=P, dD=P, ws=None, ws_bytes=0):
        return lib.sdgp_conv_bwd_data_grouped(dO, W, dD, 2, 8, 8, C_in, C_out, 3, 3, 1, 1, groups, dt, n, m, rk, 0, ws, ws_bytes, None)

    def need(groups, C_in=32, C_out=64, n=2, m=4, dt=1):
        return lib.sdgp_conv_bwd_data_grouped_workspace(2, 8, 8, C_in, C_out, 3, 3, 1, 1, groups, dt, n, m)

    bad = ctypes.c_size_t(-1).value
    assert call(0) == E_SHAPE and call(3) == E_SHAPE and call(-2) == E_SHAPE      # 32 % 3 != 0
    assert call(32, m=4) == E_SHAPE                                               # two output channels per group
    assert need(0) == bad and need(3) == bad and need(32) == bad
    assert need(4) == 2 * 8 * 8 * 64 * 2 and need(4, dt=0) == 2 * 8 * 8 * 64 * 4    # the pruned gradient
    assert need(4, n=4) == 0                                                      # dense: nothing to prune
    assert need(1) == lib.sdgp_conv_bwd_data_workspace(2, 8, 8, 32, 64, 3, 3, 1, 1, 1, 2, 4)
    assert call(4) == E_WS and call(4, ws=P, ws_bytes=need(4) - 1) == E_WS
    assert call(4, ws=P, ws_bytes=need(4), dO=None) == E_NULL
    assert call(4, rk=7, ws=P, ws_bytes=need(4)) == E_RANKER
    assert call(4, dt=5) == E_DTYPE and call(4, n=5) == E_NM


def test_peak_probe_argument_errors(lib):
    lib.sdgp_peak_probe.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                    ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    work = ctypes.c_double(0.0)
    w = ctypes.byref(work)
    assert lib.sdgp_peak_probe(0, P, P, 1024, 1, None, None) == E_NULL
    assert lib.sdgp_peak_probe(0, None, P, 1024, 1, w, None) == E_NULL
    assert lib.sdgp_peak_probe(2, None, None, 0, 1, w, None) == E_NULL
    assert lib.sdgp_peak_probe(4, P, P, 1024, 1, w, None) == E_SHAPE and lib.sdgp_peak_probe(-1, P, P, 1024, 1, w, None) == E_SHAPE
    assert lib.sdgp_peak_probe(1, ctypes.c_void_p(24), P, 1024, 1, w, None) == E_SHAPE       # not 16-byte aligned
    assert lib.sdgp_peak_probe(3, None, P, 0, 0, w, None) == E_SHAPE and lib.sdgp_peak_probe(2, None, P, 0, (1 << 20) + 1, w, None) == E_SHAPE
