"""Operand layouts of the matrix instructions and of the transposing LDS read, as the kernels assume them.

One wavefront runs one instruction on register contents laid out here from small integer matrices (exact in bf16 and
in the fp32 sums); the result registers must be the matrix product, read back through the assumed result layout.

  mfma 32x32x16 bf16:    A lane l: row l%32, k = 8*(l/32) + e (e < 8); B lane l: column l%32, same k;
                         D lane l, register r: column l%32, row 8*(r/4) + 4*(l/32) + r%4.
  mfma 16x16x32 bf16:    A lane l: row l%16, k = 8*(l/16) + e (e < 8); B lane l: column l%16, same k;
                         D lane l, register r: column l%16, row 4*(l/16) + r.
  smfmac 32x32x32 bf16:  A lane l: row l%32, 8 kept values of dense k = 16*(l/32) .. +15; value e belongs to quad e/2
                         and sits at position (idx >> 2e) & 3 of it; B lane l: column l%32, element eb:
                         k = 16*(eb/8) + 8*(l/32) + eb%8; D as above.
  ds_read_b64_tr_b16:    in each group of 16 lanes, lane i receives element i%4 of the 8 bytes addressed by lanes
                         i/4, 4 + i/4, 8 + i/4 and 12 + i/4 of the group.
"""
import ctypes
import os

import numpy as np
import pytest
import torch

from paper_2202_00774_amd import workloads as wl
from util import to_gpu

pytestmark = pytest.mark.gpu
LIB = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "libmatrix_layout_probe.so")


@pytest.fixture(scope="module")
def probe():
    assert os.path.exists(LIB), "tests/native/libmatrix_layout_probe.so is not built: run python -m paper_2202_00774_amd.build"
    lib = ctypes.CDLL(LIB)
    for name in ("layout_mfma_32x32x16_bf16", "layout_mfma_16x16x32_bf16", "layout_smfmac_32x32x32_bf16", "layout_ds_read_tr16_b64"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


def bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, np.float32))


def ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def result_matrix(d):
    """[64 lanes][16 registers] -> [32 rows][32 columns] by the assumed result layout."""
    D = np.empty((32, 32), np.float32)
    for l in range(64):
        for r in range(16):
            D[8 * (r // 4) + 4 * (l // 32) + r % 4, l % 32] = d[l, r]
    return D


def test_mfma_32x32x16_operand_layout(probe):
    rng = np.random.default_rng(1)
    A = rng.integers(-8, 9, (32, 16)).astype(np.float32)
    B = rng.integers(-8, 9, (16, 32)).astype(np.float32)
    a = np.empty((64, 8), np.float32)
    b = np.empty((64, 8), np.float32)
    for l in range(64):
        for e in range(8):
            a[l, e] = A[l % 32, 8 * (l // 32) + e]
            b[l, e] = B[8 * (l // 32) + e, l % 32]
    d = torch.zeros((64, 16), dtype=torch.float32, device="cuda")
    ta, tb = to_gpu(bf16(a)), to_gpu(bf16(b))
    assert probe.layout_mfma_32x32x16_bf16(ptr(ta), ptr(tb), ptr(d), stream()) == 0
    torch.cuda.synchronize()
    assert np.array_equal(result_matrix(d.cpu().numpy()), A @ B)


def test_mfma_16x16x32_operand_layout(probe):
    rng = np.random.default_rng(11)
    A = rng.integers(-8, 9, (16, 32)).astype(np.float32)
    B = rng.integers(-8, 9, (32, 16)).astype(np.float32)
    a = np.empty((64, 8), np.float32)
    b = np.empty((64, 8), np.float32)
    for l in range(64):
        for e in range(8):
            a[l, e] = A[l % 16, 8 * (l // 16) + e]
            b[l, e] = B[8 * (l // 16) + e, l % 16]
    d = torch.zeros((64, 4), dtype=torch.float32, device="cuda")
    ta, tb = to_gpu(bf16(a)), to_gpu(bf16(b))
    assert probe.layout_mfma_16x16x32_bf16(ptr(ta), ptr(tb), ptr(d), stream()) == 0
    torch.cuda.synchronize()
    got = d.cpu().numpy()
    D = np.empty((16, 16), np.float32)
    for l in range(64):
        for r in range(4):
            D[4 * (l // 16) + r, l % 16] = got[l, r]
    assert np.array_equal(D, A @ B)


@pytest.mark.parametrize("seed", [2, 3])
def test_smfmac_32x32x32_operand_layout(probe, seed):
    rng = np.random.default_rng(seed)
    A = np.zeros((32, 32), np.float32)            # two nonzeros in every aligned quad of k
    a = np.zeros((64, 8), np.float32)
    idx = np.zeros(64, np.uint32)
    for l in range(64):
        row, k0 = l % 32, 16 * (l // 32)
        for quad in range(4):
            pos = np.sort(rng.choice(4, 2, replace=False))
            for j in range(2):
                e = 2 * quad + j
                v = float(rng.integers(1, 9) * rng.choice([-1, 1]))
                A[row, k0 + 4 * quad + pos[j]] = v
                a[l, e] = v
                idx[l] |= np.uint32(int(pos[j]) << (2 * e))
    B = rng.integers(-8, 9, (32, 32)).astype(np.float32)
    b = np.empty((64, 16), np.float32)
    for l in range(64):
        for eb in range(16):
            b[l, eb] = B[16 * (eb // 8) + 8 * (l // 32) + eb % 8, l % 32]
    d = torch.zeros((64, 16), dtype=torch.float32, device="cuda")
    ta, tb = to_gpu(bf16(a)), to_gpu(bf16(b))
    ti = torch.from_numpy(idx.view(np.int32)).cuda()
    assert probe.layout_smfmac_32x32x32_bf16(ptr(ta), ptr(ti), ptr(tb), ptr(d), stream()) == 0
    torch.cuda.synchronize()
    assert np.array_equal(result_matrix(d.cpu().numpy()), A @ B)


def test_smfmac_first_slot_may_hold_a_dropped_position(probe):
    """A quad with one survivor: the empty slot carries value +0 and a dropped position, on either side of the survivor."""
    A = np.zeros((32, 32), np.float32)
    a = np.zeros((64, 8), np.float32)
    idx = np.zeros(64, np.uint32)
    for l in range(64):
        row, k0 = l % 32, 16 * (l // 32)
        for quad in range(4):
            keep = (row + quad) % 4                 # one survivor per quad, at a position that moves
            other = (keep + 1 + row % 3) % 4        # the empty slot names some dropped position
            v = float(1 + (row + quad) % 7)
            A[row, k0 + 4 * quad + keep] = v
            lo, hi = min(keep, other), max(keep, other)
            a[l, 2 * quad + (0 if keep == lo else 1)] = v
            idx[l] |= np.uint32((lo << (4 * quad)) | (hi << (4 * quad + 2)))
    B = np.random.default_rng(5).integers(-8, 9, (32, 32)).astype(np.float32)
    b = np.empty((64, 16), np.float32)
    for l in range(64):
        for eb in range(16):
            b[l, eb] = B[16 * (eb // 8) + 8 * (l // 32) + eb % 8, l % 32]
    d = torch.zeros((64, 16), dtype=torch.float32, device="cuda")
    ta, tb = to_gpu(bf16(a)), to_gpu(bf16(b))
    ti = torch.from_numpy(idx.view(np.int32)).cuda()
    assert probe.layout_smfmac_32x32x32_bf16(ptr(ta), ptr(ti), ptr(tb), ptr(d), stream()) == 0
    torch.cuda.synchronize()
    assert np.array_equal(result_matrix(d.cpu().numpy()), A @ B)


def test_transposing_lds_read_lane_exchange(probe):
    words = 1024
    data = np.arange(words, dtype=np.uint16) * 3 + 1
    rng = np.random.default_rng(7)
    addr = (rng.permutation(words // 4)[:64] * 8).astype(np.uint32)      # distinct 8-byte slots
    out = torch.zeros((64, 4), dtype=torch.int16, device="cuda")
    tin = torch.from_numpy(data.view(np.int16)).cuda()
    assert probe.layout_ds_read_tr16_b64(ptr(tin), words, addr.ctypes.data_as(ctypes.c_void_p), ptr(out), stream()) == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    want = np.empty((64, 4), np.uint16)
    for lane in range(64):
        g, i = lane // 16 * 16, lane % 16
        for j in range(4):
            src = g + 4 * j + i // 4
            want[lane, j] = data[addr[src] // 2 + i % 4]
    assert np.array_equal(got, want)
    # a B fragment straight from a row-major [k][n] slab: lane L addresses row L/4, columns 4*(L%4)..; lane i of the
    # group then holds column i for four consecutive k
    pitch = 16                                                            # one 16-lane group: 4 rows x 16 columns
    addr2 = np.array([((l % 16) // 4 * pitch + 4 * (l % 4)) * 2 + (l // 16) * 4 * pitch * 2 for l in range(64)], np.uint32)
    assert probe.layout_ds_read_tr16_b64(ptr(tin), words, addr2.ctypes.data_as(ctypes.c_void_p), ptr(out), stream()) == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    for lane in range(64):
        base = lane // 16 * 4 * pitch
        assert got[lane].tolist() == [int(data[base + k * pitch + lane % 16]) for k in range(4)]

    bad = addr.copy()
    bad[5] = words * 2                                                    # outside the array: refused on the host
    assert probe.layout_ds_read_tr16_b64(ptr(tin), words, bad.ctypes.data_as(ctypes.c_void_p), ptr(out), stream()) == 2
