// Pieces shared by the matrix-core backward-data kernels that move data with direct-to-LDS loads:
// the copy itself (global_load_lds_dwordx4), the counter wait, and the ranking of sixteen channels of one gradient
// pixel into the operand of the structured-sparse matrix instruction (Sec. III-B).
#pragma once

#include "bwd_tiled.h"

namespace sdgp {

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_base + 16*i.  The compiler does not see
// these as memory instructions; callers wait with wait_lds_copies.
__device__ __forceinline__ void lds_copy16(const void* gptr, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);  // wave-uniform by construction
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(gptr) : "memory");
}
// Four bytes per lane: lane l's word lands at lds_base + 4 l.
__device__ __forceinline__ void lds_copy4(const void* gptr, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(base), "v"(gptr) : "memory");
}
// Same, address = wave-uniform base + 32-bit byte offset per lane.
__device__ __forceinline__ void lds_copy16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
    const uint64_t a = (uint64_t)(uintptr_t)sbase;
    // (the builtin returns a signed int: go through uint32_t, or the low word sign-extends into the high one)
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
    const uint64_t ua = ((uint64_t)hi << 32) | (uint64_t)lo;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(base), "v"(voff), "s"(ua) : "memory");
}
// Waits until at most N of this wavefront's vector-memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wait_lds_copies() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Sixteen consecutive channels of one gradient pixel -> the compressed operand (Sec. III-B).
template <int M, int RK>
__device__ __forceinline__ void prune16_compressed(const u32x4_t (&v)[2], int n, uint32_t mix, uint64_t e0, uint32_t (&packed)[4],
                                             uint32_t& meta) {
    const uint32_t w[8] = {v[0][0], v[0][1], v[0][2], v[0][3], v[1][0], v[1][1], v[1][2], v[1][3]};
    prune_compress16<M, RK>(w, n, mix, e0, packed, meta);
}

// Sixteen consecutive channels of one gradient pixel, pruned (Sec. III-B) and written back dense with zeros.
// v[0], v[1]: the two 16-byte halves; e0: flat index of the first element (for the random ranker's hash).
template <int M, int RK, bool NLE2>
__device__ __forceinline__ void prune16_dense(u32x4_t (&v)[2], int n, uint32_t mix, uint64_t e0) {
    if constexpr (M == 16 && !NLE2 && RK != kRandom) {
        // one group, magnitude keys, any n: the packed 16-bit ranker, no unpacking
        const uint32_t w[8] = {v[0][0], v[0][1], v[0][2], v[0][3], v[1][0], v[1][1], v[1][2], v[1][3]};
        uint32_t o[8];
        prune_packed<16, RK>(w, n, o);
        v[0] = u32x4_t{o[0], o[1], o[2], o[3]}, v[1] = u32x4_t{o[4], o[5], o[6], o[7]};
        return;
    }
    uint32_t raw[16], out[16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            raw[i * 8 + 2 * x] = v[i][x] & 0xFFFFu;
            raw[i * 8 + 2 * x + 1] = v[i][x] >> 16;
        }
#pragma unroll
    for (int g = 0; g < 16 / M; ++g) {
        uint32_t r[M], o[M];
        bool kk[M];
#pragma unroll
        for (int j = 0; j < M; ++j) r[j] = raw[g * M + j];
        const uint64_t eg = e0 + (uint64_t)(g * M);
        prune_group<kBF16, M, RK, NLE2>(r, n, hash_row(mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
        for (int j = 0; j < M; ++j) out[g * M + j] = o[j];
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int x = 0; x < 4; ++x) v[i][x] = out[i * 8 + 2 * x] | (out[i * 8 + 2 * x + 1] << 16);
}

}  // namespace sdgp
