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

// The compressed operand of sixteen channels as a value (four dwords of kept pairs and sixteen bits of positions).
struct Packed16 {
    uint32_t p0, p1, p2, p3, meta;
};

// Random ranker, generic path: exact for any hashes.  Reached only when the key-based path cannot be sure (two hashes
// of a group agreeing in 28 bits at the threshold: about four groups in a billion), so it is kept out of line --
// inlined, its registers spilled the callers' main loops (256 to 448 bytes of scratch per lane at m = 8 and 16).
template <int M>
__device__ __attribute__((noinline)) Packed16 prune16_random_generic(u32x4_t v0, u32x4_t v1, int n, uint32_t mix, uint64_t e0) {
    const u32x4_t v[2] = {v0, v1};
    uint32_t raw[16], out[16];
    bool keep[16];
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
        prune_group<kBF16, M, kRandom, true>(r, n, hash_row(mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
        for (int j = 0; j < M; ++j) out[g * M + j] = o[j], keep[g * M + j] = kk[j];
    }
    uint32_t packed[4], meta = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bool kq[4] = {keep[4 * q], keep[4 * q + 1], keep[4 * q + 2], keep[4 * q + 3]};
        const uint32_t oq[4] = {out[4 * q], out[4 * q + 1], out[4 * q + 2], out[4 * q + 3]};
        uint32_t x0, x1, pos;
        compress_quad(kq, oq, x0, x1, pos);
        packed[q] = x0 | (x1 << 16);
        meta |= pos << (4 * q);
    }
    return {packed[0], packed[1], packed[2], packed[3], meta};
}

// Sixteen consecutive channels of one gradient pixel -> the compressed operand (Sec. III-B).
template <int M, int RK>
__device__ __forceinline__ void prune16_compressed(const u32x4_t (&v)[2], int n, uint32_t mix, uint64_t e0, uint32_t (&packed)[4],
                                             uint32_t& meta) {
    const uint32_t w[8] = {v[0][0], v[0][1], v[0][2], v[0][3], v[1][0], v[1][1], v[1][2], v[1][3]};
    if constexpr (RK != kRandom) {
        prune_compress16_bf16<M, RK>(w, n, packed, meta);
    } else {
        // fast path; it says when it cannot be sure
        bool exact;
        prune_compress16_random<M>(w, n, mix, e0, packed, meta, exact);
        if (!exact) {
            const Packed16 r = prune16_random_generic<M>(v[0], v[1], n, mix, e0);
            packed[0] = r.p0, packed[1] = r.p1, packed[2] = r.p2, packed[3] = r.p3, meta = r.meta;
        }
    }
}

#ifdef SDGP_TRACE
#define SDGP_EXP(bit) (p.exp & (bit))
#else
#define SDGP_EXP(bit) false
#endif

}  // namespace sdgp
