// One pass over the gradient that ranks every group (Alg. 1, Sec. III-B) and writes what the structured-sparse matrix
// instruction reads: per row and 16 channels the eight kept values (two per aligned quad: every n <= 2 pattern of
// m = 4, 8 or 16 fits) and one 16-bit word of 2-bit positions.  The pointwise kernel's MODE 3 multiplies from these
// without ranking anything.  Worth a pass of its own where the fused kernel would rank a gradient element many times:
// a 1x1 layer with many column tiles (every workgroup of a row tile ranks the rows itself) and strided filters (once
// per tap and parity class).
//   vals [rows][C_out / 2] bf16: row r, item i (16 channels) at r * C_out / 2 + 8 i
//   meta [C_out / 64][rows][4] uint16: the four items of a 64-channel chunk side by side, rows contiguous per chunk
#include "lds_copy.h"

namespace sdgp {

namespace {

template <int M, int RK>
__global__ void __launch_bounds__(256) compress_rows(const uint16_t* __restrict__ dO, uint32_t nitems, uint32_t ipr, int64_t rows,
                                                     int n, uint32_t mix, uint16_t* __restrict__ vals, uint16_t* __restrict__ meta) {
    const uint32_t it = blockIdx.x * 256u + threadIdx.x;
    if (it >= nitems) return;
    const uint32_t row = it / ipr, item = it - row * ipr;
    const u32x4_t* src = reinterpret_cast<const u32x4_t*>(dO) + (size_t)it * 2;
    const u32x4_t v[2] = {__builtin_nontemporal_load(src), __builtin_nontemporal_load(src + 1)};
    uint32_t packed[4], mt;
    prune16_compressed<M, RK>(v, n, mix, (uint64_t)it * 16u, packed, mt);
    const u32x4_t x = {packed[0], packed[1], packed[2], packed[3]};
    *(reinterpret_cast<u32x4_t*>(vals) + it) = x;
    meta[((size_t)(item >> 2) * (size_t)rows + row) * 4u + (item & 3u)] = (uint16_t)mt;
}

template <int M>
int compress_launch_m(const uint16_t* dO, uint32_t nitems, uint32_t ipr, int64_t rows, int n, int rk, uint32_t mix, uint16_t* vals,
                      uint16_t* meta, hipStream_t stream) {
    const dim3 grid((nitems + 255u) / 256u), block(256);
    if (rk == kRandom) hipLaunchKernelGGL((compress_rows<M, kRandom>), grid, block, 0, stream, dO, nitems, ipr, rows, n, mix, vals, meta);
    else if (rk == kGreedy) hipLaunchKernelGGL((compress_rows<M, kGreedy>), grid, block, 0, stream, dO, nitems, ipr, rows, n, mix, vals, meta);
    else hipLaunchKernelGGL((compress_rows<M, kAdjusted>), grid, block, 0, stream, dO, nitems, ipr, rows, n, mix, vals, meta);
    return launch_status();
}

}  // namespace

// Bytes of the two arrays for a gradient of rows x C_out (C_out a multiple of 64); the positions start at
// compress_meta_offset.
size_t compress_meta_offset(int64_t rows, int64_t C_out) { return ((size_t)rows * (size_t)C_out + 255u) & ~(size_t)255u; }
size_t compress_bytes(int64_t rows, int64_t C_out) { return compress_meta_offset(rows, C_out) + (size_t)rows * (size_t)(C_out / 64) * 8u; }

// dO [rows][C_out] bf16, n <= 2 of m in {4, 8, 16}, C_out a multiple of 64, rows * C_out / 16 < 2^31, 16-byte aligned
// pointers (the callers check).  The flat element index of the random ranker is row * C_out + channel, as everywhere.
int compress_launch(const void* dO, int64_t rows, int64_t C_out, int n, int m, int rk, uint64_t seed, void* workspace,
                    hipStream_t stream) {
    const uint32_t ipr = (uint32_t)(C_out / 16), nitems = (uint32_t)(rows * (C_out / 16));
    uint16_t* vals = static_cast<uint16_t*>(workspace);
    uint16_t* meta = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(workspace) + compress_meta_offset(rows, C_out));
    const uint16_t* src = static_cast<const uint16_t*>(dO);
    const uint32_t mix = seed_mix(seed);
    if (m == 4) return compress_launch_m<4>(src, nitems, ipr, rows, n, rk, mix, vals, meta, stream);
    if (m == 8) return compress_launch_m<8>(src, nitems, ipr, rows, n, rk, mix, vals, meta, stream);
    return compress_launch_m<16>(src, nitems, ipr, rows, n, rk, mix, vals, meta, stream);
}

}  // namespace sdgp
