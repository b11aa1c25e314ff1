// The pruning function P of Sec. III-B applied to one group of M channels held
// in registers.  Used by the standalone prune kernel and by the fused
// backward-data kernels, so both produce identical bits.
//
// Ranking is integer work.  The kept set is the n positions with the largest
// (key, -position): key = |x| as the sign-cleared bit pattern (Magnitude and
// Rescaled Magnitude) or the counter hash of the flat element index (Random).
// Rescaled Magnitude multiplies the kept values by S/T, S = sum |x| over the
// group, T = sum |x| over the kept, both accumulated in fp32 in ascending
// position, one IEEE division, then rounds the product to the storage type.
#pragma once

#include "common.h"

namespace sdgp {

enum : int { kF32 = SDGP_F32, kBF16 = SDGP_BF16 };
enum : int { kRandom = SDGP_RANDOM, kGreedy = SDGP_GREEDY, kAdjusted = SDGP_GREEDY_ADJUSTED };

// Median of three unsigned values (the compiler folds this into v_med3_u32).
__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
    return max(min(a, b), min(max(a, b), c));
}

// Pairwise rank count: rank[j] = number of elements that beat j, where a lower
// position wins ties.  keep[j] = rank[j] < n.  Exact for any keys and any n.
template <int M>
__device__ __forceinline__ void select_by_rank(const uint32_t (&key)[M], int n, bool (&keep)[M]) {
    int rank[M];
#pragma unroll
    for (int j = 0; j < M; ++j) rank[j] = j;  // every lower position beats j unless j's key is strictly larger
#pragma unroll
    for (int a = 0; a < M; ++a) {
#pragma unroll
        for (int b = a + 1; b < M; ++b) {
            const bool g = key[b] > key[a];  // b beats a only when strictly larger
            rank[a] += g ? 1 : 0;
            rank[b] -= g ? 1 : 0;
        }
    }
#pragma unroll
    for (int j = 0; j < M; ++j) keep[j] = rank[j] < n;
}

// n <= 2, keys pairwise distinct: the threshold is the largest or second
// largest key, found with one max and one median per element.
template <int M>
__device__ __forceinline__ void select_top2_distinct(const uint32_t (&key)[M], int n, bool (&keep)[M]) {
    uint32_t v1 = key[0], v2 = 0;
    if constexpr (M > 1) {
        v1 = max(key[0], key[1]);
        v2 = min(key[0], key[1]);
    }
#pragma unroll
    for (int j = 2; j < M; ++j) {
        v2 = umed3(v1, v2, key[j]);
        v1 = max(v1, key[j]);
    }
    const uint32_t thr = (n == 1 || M == 1) ? v1 : v2;
#pragma unroll
    for (int j = 0; j < M; ++j) keep[j] = key[j] >= thr;
}

// n <= 2, keys may repeat: track the three largest keys as a multiset.  Only
// when the threshold key is shared by a key that must be dropped does position
// decide, and then the exact rank count takes over (rare for hash keys).
template <int M>
__device__ __forceinline__ void select_top2_ties(const uint32_t (&key)[M], int n, bool (&keep)[M]) {
    static_assert(M >= 3, "needs at least three keys");
    uint32_t v1 = max(key[0], key[1]);
    uint32_t v2 = min(key[0], key[1]);
    uint32_t v3 = min(v2, key[2]);
    v2 = umed3(v1, v2, key[2]);
    v1 = max(v1, key[2]);
#pragma unroll
    for (int j = 3; j < M; ++j) {
        v3 = umed3(v2, v3, key[j]);
        v2 = umed3(v1, v2, key[j]);
        v1 = max(v1, key[j]);
    }
    const bool tie = (n == 1) ? (v1 == v2) : (v2 == v3);
    if (tie) {
        select_by_rank<M>(key, n, keep);
    } else {
        const uint32_t thr = (n == 1) ? v1 : v2;
#pragma unroll
        for (int j = 0; j < M; ++j) keep[j] = key[j] >= thr;
    }
}

// One group.
//   raw[j]   stored bit pattern of element j (16 significant bits for bf16)
//   n        elements to keep, 1 <= n <= M
//   hrow     hash_row(mix, high word of the group's flat index)   (Random only)
//   e_lo     low word of the flat index of element 0              (Random only)
//   NLE2     compile-time promise that n <= 2 (enables the threshold selects)
// Output: keep[j], and out[j] = stored bit pattern of the pruned element
// (+0 where dropped).
template <int DT, int M, int RK, bool NLE2>
__device__ __forceinline__ void prune_group(const uint32_t (&raw)[M], int n, uint32_t hrow, uint32_t e_lo,
                                            bool (&keep)[M], uint32_t (&out)[M]) {
    constexpr uint32_t kMagMask = (DT == kBF16) ? 0x7FFFu : 0x7FFFFFFFu;
    uint32_t key[M];
    if constexpr (RK == kRandom) {
#pragma unroll
        for (int j = 0; j < M; ++j) key[j] = hash_elem(hrow, e_lo + (uint32_t)j);
    } else {
#pragma unroll
        for (int j = 0; j < M; ++j) key[j] = raw[j] & kMagMask;
    }

    if constexpr (M == 1) {
        keep[0] = true;
    } else if constexpr (RK != kRandom && DT == kBF16) {
        // 15-bit magnitudes: fold the position in to make the keys distinct,
        // a lower position giving the larger key.
#pragma unroll
        for (int j = 0; j < M; ++j) key[j] = (key[j] << 5) | (uint32_t)(31 - j);
        if constexpr (NLE2) select_top2_distinct<M>(key, n, keep);
        else select_by_rank<M>(key, n, keep);
    } else if constexpr (NLE2 && M >= 8) {
        select_top2_ties<M>(key, n, keep);
    } else {
        select_by_rank<M>(key, n, keep);
    }

    if constexpr (RK == kAdjusted) {
        float total = 0.0f, kept = 0.0f;
        float x[M];
#pragma unroll
        for (int j = 0; j < M; ++j) {
            x[j] = (DT == kBF16) ? bf16_to_float(raw[j]) : bits_to_float(raw[j]);
            const float a = bits_to_float(float_to_bits(x[j]) & 0x7FFFFFFFu);
            total = __fadd_rn(total, a);
            kept = keep[j] ? __fadd_rn(kept, a) : kept;
        }
        const float scale = (kept == 0.0f) ? 1.0f : __fdiv_rn(total, kept);
#pragma unroll
        for (int j = 0; j < M; ++j) {
            const float y = __fmul_rn(x[j], scale);
            const uint32_t yb = (DT == kBF16) ? float_to_bf16(y) : float_to_bits(y);
            out[j] = keep[j] ? yb : 0u;
        }
    } else {
#pragma unroll
        for (int j = 0; j < M; ++j) out[j] = keep[j] ? raw[j] : 0u;
    }
}

}  // namespace sdgp
