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
__host__ __device__ __forceinline__ void select_by_rank(const uint32_t (&key)[M], int n, bool (&keep)[M]) {
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

// Any n, keys pairwise distinct: sort a copy of the keys (bitonic network, M/2 * log2(M) * (log2(M) + 1) / 2
// compare-exchanges of one min and one max: 80 for sixteen keys, 240 for thirty-two -- a third of the rank count's
// instructions, and no rank registers), take the n-th largest as the threshold.
template <int M>
__device__ __forceinline__ void select_by_sort(const uint32_t (&key)[M], int n, bool (&keep)[M]) {
    static_assert((M & (M - 1)) == 0 && M >= 2, "power of two");
    uint32_t s[M];
#pragma unroll
    for (int j = 0; j < M; ++j) s[j] = key[j];
#pragma unroll
    for (int k = 2; k <= M; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int i = 0; i < M; ++i) {
                const int l = i ^ j;
                if (l > i) {
                    const uint32_t a = s[i], b = s[l];
                    const bool desc = (i & k) == 0;  // descending runs first: s[0] ends up the largest
                    s[i] = desc ? max(a, b) : min(a, b);
                    s[l] = desc ? min(a, b) : max(a, b);
                }
            }
        }
    }
    uint32_t thr = s[0];
#pragma unroll
    for (int i = 1; i < M; ++i) thr = (i == n - 1) ? s[i] : thr;  // n is wavefront-uniform: scalar selects
#pragma unroll
    for (int j = 0; j < M; ++j) keep[j] = key[j] >= thr;
}

// Any n, keys that rarely repeat (hash keys of a group too wide for a position code): the sorting network again.  With
// s the keys in descending order, the kept set is {key >= s[n-1]} unless the key after the threshold equals it -- only
// then does position decide between equal keys, and the exact rank count takes over (about one group of 32 in a
// million for 28-bit hash keys).
template <int M>
__host__ __device__ __forceinline__ void select_by_sort_ties(const uint32_t (&key)[M], int n, bool (&keep)[M]) {
    static_assert((M & (M - 1)) == 0 && M >= 2, "power of two");
    uint32_t s[M];
#pragma unroll
    for (int j = 0; j < M; ++j) s[j] = key[j];
#pragma unroll
    for (int k = 2; k <= M; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int i = 0; i < M; ++i) {
                const int l = i ^ j;
                if (l > i) {
                    const uint32_t a = s[i], b = s[l];
                    const uint32_t hi = a > b ? a : b, lo = a > b ? b : a;
                    const bool desc = (i & k) == 0;  // descending runs first: s[0] ends up the largest
                    s[i] = desc ? hi : lo;
                    s[l] = desc ? lo : hi;
                }
            }
        }
    }
    uint32_t thr = s[0], next = 0;
    bool has_next = false;
#pragma unroll
    for (int i = 1; i < M; ++i) {   // n is wavefront-uniform: scalar selects
        thr = (i == n - 1) ? s[i] : thr;
        next = (i == n) ? s[i] : next;
        has_next = has_next || i == n;
    }
    if (has_next && next == thr) {
        select_by_rank<M>(key, n, keep);
        return;
    }
#pragma unroll
    for (int j = 0; j < M; ++j) keep[j] = key[j] >= thr;
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
//   SORT     any n on distinct keys: sorting network (fewer instructions: the fused kernels) or rank count (measured
//            faster in the streaming prune kernel)
// Output: keep[j], and out[j] = stored bit pattern of the pruned element
// (+0 where dropped).
template <int DT, int M, int RK, bool NLE2, bool SORT = true>
__device__ __forceinline__ void prune_group(const uint32_t (&raw)[M], int n, uint32_t hrow, uint32_t e_lo,
                                            bool (&keep)[M], uint32_t (&out)[M]) {
    constexpr uint32_t kMagMask = (DT == kBF16) ? 0x7FFFu : 0x7FFFFFFFu;
    uint32_t key[M];
    if constexpr (RK == kRandom && M % 4 == 0) {
        // a group starts at a multiple of M, so its quads are the hash's quads: one mixed word each
#pragma unroll
        for (int q = 0; q < M / 4; ++q) {
            const uint32_t hq = hash_quad(hrow, e_lo + 4u * (uint32_t)q);
#pragma unroll
            for (int i = 0; i < 4; ++i) key[4 * q + i] = hash_lane(hq, (uint32_t)i);
        }
    } else if constexpr (RK == kRandom) {
#pragma unroll
        for (int j = 0; j < M; ++j) key[j] = hash_elem(hrow, e_lo + (uint32_t)j);
    } else {
#pragma unroll
        for (int j = 0; j < M; ++j) key[j] = raw[j] & kMagMask;
    }

    if constexpr (M == 1) {
        keep[0] = true;
    } else if constexpr ((RK != kRandom && DT == kBF16) || (RK == kRandom && M <= 16)) {
        // 15-bit magnitudes, and hash keys (28 bits wide, their low four bits clear) of groups up to 16: fold the
        // position in to make the keys distinct, a lower position giving the larger key.
#pragma unroll
        for (int j = 0; j < M; ++j) key[j] = RK == kRandom ? (key[j] | (uint32_t)(15 - j)) : ((key[j] << 5) | (uint32_t)(31 - j));
        if constexpr (NLE2) select_top2_distinct<M>(key, n, keep);
        else if constexpr (SORT && M >= 8 && (M & (M - 1)) == 0) select_by_sort<M>(key, n, keep);
        else select_by_rank<M>(key, n, keep);
    } else if constexpr (NLE2 && M >= 16) {
        // (for eight keys the 28 comparisons of the rank count measured faster than the multiset and its fallback)
        select_top2_ties<M>(key, n, keep);
    } else if constexpr (RK == kRandom && M == 32) {
        select_by_sort_ties<M>(key, n, keep);
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
        if constexpr (DT == kBF16 && M % 2 == 0) {
#pragma unroll
            for (int j = 0; j < M; j += 2) {
                const uint32_t yb = float2_to_bf16x2(__fmul_rn(x[j], scale), __fmul_rn(x[j + 1], scale));
                out[j] = keep[j] ? (yb & 0xFFFFu) : 0u;
                out[j + 1] = keep[j + 1] ? (yb >> 16) : 0u;
            }
        } else {
#pragma unroll
            for (int j = 0; j < M; ++j) {
                const float y = __fmul_rn(x[j], scale);
                const uint32_t yb = (DT == kBF16) ? float_to_bf16(y) : float_to_bits(y);
                out[j] = keep[j] ? yb : 0u;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < M; ++j) out[j] = keep[j] ? raw[j] : 0u;
    }
}

// Magnitude / Rescaled Magnitude with n <= 2 on sixteen consecutive bf16 channels (eight dwords, channel 2i in
// the low half of dword i), producing the operand format of the structured-sparse matrix instructions directly:
// per aligned quad of channels two values (lower position in the low half of the output dword) and two 2-bit
// positions, ascending, four bits per quad in `meta`.  A slot without a survivor holds +0 and points at a
// dropped position.  Bit-identical to prune_group followed by a compaction, at about half the instructions.
//
// Every element becomes one 32-bit key: magnitude in bits 17..31, a "kept" mark in bit 9, (M-1 - position in
// group) in bits 1..4, sign in bit 0.  Keys are distinct, a lower position wins equal magnitudes (Sec. III-B
// reading: stable ties), and a key carries everything needed to rebuild its value.  The two largest keys of a
// quad contain every survivor of that quad; the group's threshold is the n-th largest key over its quads.
// Rotated right by nine bits a key reads [code | sign | magnitude | mark]: unsigned order is now position order
// and the bf16 value sits byte-aligned in bits 8..23.
// ---- Magnitude / Rescaled Magnitude on a group of 16 or 32 bf16 channels, any n, on packed 16-bit arithmetic.
// A dword carries two magnitudes and the packed instructions (max, min, saturating subtract) treat both at once:
//   1. the magnitudes are sorted by a bitonic network whose slot s is half s / (M/2) of dword s % (M/2) -- a stage
//      pairs whole dwords (one packed max and one packed min for two compare-exchanges) except the one stage whose
//      partner is the other half of the same dword; the network only needs the values, not where they came from;
//   2. the threshold T is the n-th largest magnitude; an element is kept when its magnitude exceeds T, or equals T
//      and fewer than n - #(greater) equal elements precede it (the lower position wins: Sec. III-B reading), all of it
//      as 0/1 arithmetic on halves: [a > T] = min(a -sat T, 1), [a == T] = 1 -sat (a xor T), a running count of
//      equals in position order.
// About 20 instructions per element at M = 32 where the pairwise rank count takes about 46.
typedef uint16_t sdgp_u16x2 __attribute__((ext_vector_type(2)));
__host__ __device__ __forceinline__ uint32_t sdgp_max_u32(uint32_t a, uint32_t b) { return a > b ? a : b; }
__host__ __device__ __forceinline__ uint32_t sdgp_min_u32(uint32_t a, uint32_t b) { return a < b ? a : b; }
__host__ __device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(sdgp_u16x2, a), __builtin_bit_cast(sdgp_u16x2, b)));
}
__host__ __device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(sdgp_u16x2, a), __builtin_bit_cast(sdgp_u16x2, b)));
}
__host__ __device__ __forceinline__ uint32_t pk_sub_sat(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(__builtin_bit_cast(sdgp_u16x2, a), __builtin_bit_cast(sdgp_u16x2, b)));
}
__host__ __device__ __forceinline__ uint32_t pk_add(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, (sdgp_u16x2)(__builtin_bit_cast(sdgp_u16x2, a) + __builtin_bit_cast(sdgp_u16x2, b)));
}
__host__ __device__ __forceinline__ uint32_t pk_neg(uint32_t a) {   // 0 -> 0, 1 -> 0xFFFF per half
    return __builtin_bit_cast(uint32_t, (sdgp_u16x2)(-__builtin_bit_cast(sdgp_u16x2, a)));
}

__host__ __device__ __forceinline__ uint32_t pk_mul(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, (sdgp_u16x2)(__builtin_bit_cast(sdgp_u16x2, a) * __builtin_bit_cast(sdgp_u16x2, b)));
}
// c + low half of a + high half of a
__host__ __device__ __forceinline__ uint32_t pk_sum_into(uint32_t a, uint32_t c) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_sad_u16(a, 0u, c);
#else
    return c + (a & 0xFFFFu) + (a >> 16);
#endif
}

// The n-th largest of M 15-bit magnitudes, two per dword (any assignment of values to halves).
//   n <= M/2: both halves of the dwords are sorted at once (two descending runs of M/2), the M/2 largest of the union
//             are max(low run[r], high run[M/2-1-r]) -- a bitonic sequence -- and one merge orders them;
//   n >  M/2: the whole network (the one stage whose partner is the other half of the same dword costs four
//             instructions per dword).
template <int M>
__host__ __device__ __forceinline__ uint32_t nth_largest_packed(const uint32_t (&mag)[M / 2], int n) {
    constexpr int R = M / 2;
    uint32_t s[R];
#pragma unroll
    for (int i = 0; i < R; ++i) s[i] = mag[i];
    // slot t = half t / R of s[t % R]; runs of length k, descending where (slot & k) == 0.  With `both_down` every
    // run of length R is descending in both halves (two independent sorts of R values).
    auto stage = [&](int k, int j, bool both_down) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int l = r ^ j;
            if (l > r) {
                const uint32_t hi = pk_max(s[r], s[l]), lo = pk_min(s[r], s[l]);
                const bool desc_low = (r & k) == 0, desc_high = both_down ? desc_low : ((r + R) & k) == 0;
                const uint32_t first_low = desc_low ? hi : lo, first_high = desc_high ? hi : lo;
                const uint32_t second_low = desc_low ? lo : hi, second_high = desc_high ? lo : hi;
                s[r] = desc_low == desc_high ? first_low : ((first_low & 0xFFFFu) | (first_high & 0xFFFF0000u));
                s[l] = desc_low == desc_high ? second_low : ((second_low & 0xFFFFu) | (second_high & 0xFFFF0000u));
            }
        }
    };
    uint32_t thr;
    if (n <= R) {
#pragma unroll
        for (int k = 2; k <= R; k <<= 1)
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1) stage(k, j, true);
        uint32_t top[R];   // the R largest, one per dword (low half; the high half is zero)
#pragma unroll
        for (int r = 0; r < R; ++r) top[r] = sdgp_max_u32(s[r] & 0xFFFFu, s[R - 1 - r] >> 16);
#pragma unroll
        for (int j = R >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int l = r ^ j;
                if (l > r) {
                    const uint32_t hi = sdgp_max_u32(top[r], top[l]), lo = sdgp_min_u32(top[r], top[l]);
                    top[r] = hi, top[l] = lo;
                }
            }
        }
        thr = top[0];
#pragma unroll
        for (int r = 1; r < R; ++r) thr = (n - 1 == r) ? top[r] : thr;
    } else {
#pragma unroll
        for (int k = 2; k <= M; k <<= 1) {
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1) {
                if (j == R) {
                    // partner = the other half of the same dword; both slots lie in a descending run (k == M)
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const uint32_t a = s[r], b = (a << 16) | (a >> 16);
                        s[r] = (pk_max(a, b) & 0xFFFFu) | (pk_min(a, b) & 0xFFFF0000u);
                    }
                } else {
                    stage(k, j, false);
                }
            }
        }
        thr = s[0];
#pragma unroll
        for (int r = 1; r < R; ++r) thr = ((n - 1) % R == r) ? s[r] : thr;
        thr = thr >> 16;   // slots R .. M-1 are the high halves
    }
    return thr;
}

// w: M bf16 channels, channel 2i in the low half of w[i].  keep[i]: 1 in the halves of the kept channels, else 0.
template <int M>
__host__ __device__ __forceinline__ void keep_flags_packed(const uint32_t (&w)[M / 2], int n, uint32_t (&keep)[M / 2]) {
    static_assert(M == 16 || M == 32, "two or four 16-byte vectors");
    constexpr int R = M / 2;
    constexpr uint32_t kOne = 0x00010001u;
    uint32_t mag[R];
#pragma unroll
    for (int i = 0; i < R; ++i) mag[i] = w[i] & 0x7FFF7FFFu;
    uint32_t thr = nth_largest_packed<M>(mag, n);   // (n is uniform over the wavefront: one branch)
    thr |= thr << 16;

    uint32_t gt[R], eq[R], greater = 0;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        gt[i] = pk_min(pk_sub_sat(mag[i], thr), kOne);
        eq[i] = pk_sub_sat(kOne, mag[i] ^ thr);
        greater = pk_sum_into(gt[i], greater);
    }
    uint32_t quota = (uint32_t)n - greater;   // equals still to be kept: at least one
    quota |= quota << 16;
    uint32_t before = 0;                      // equals at lower positions
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const uint32_t seen = pk_add(before | (before << 16), eq[i] << 16);      // the high half also follows the low one
        const uint32_t room = pk_min(pk_sub_sat(quota, seen), kOne);            // [seen < quota]
        keep[i] = gt[i] | (eq[i] & room);
        before = pk_sum_into(eq[i], before);
    }
}

// The same as masks: 0xFFFF in the halves of the kept channels.
template <int M>
__host__ __device__ __forceinline__ void keep_mask_packed(const uint32_t (&w)[M / 2], int n, uint32_t (&mask)[M / 2]) {
    uint32_t keep[M / 2];
    keep_flags_packed<M>(w, n, keep);
#pragma unroll
    for (int i = 0; i < M / 2; ++i) mask[i] = pk_neg(keep[i]);
}

// Alg. 1 on one group of M = 16 or 32 bf16 channels (two per dword), Magnitude or Rescaled Magnitude, any n: the
// pruned group in the same packing (+0 where dropped).  Bit-identical to prune_group.
template <int M, int RK>
__host__ __device__ __forceinline__ void prune_packed(const uint32_t (&w)[M / 2], int n, uint32_t (&o)[M / 2]) {
    static_assert(RK == kGreedy || RK == kAdjusted, "magnitude keys");
    uint32_t flag[M / 2];
    keep_flags_packed<M>(w, n, flag);
    if constexpr (RK == kAdjusted) {
        float total = 0.0f, kept = 0.0f, x[M];
#pragma unroll
        for (int j = 0; j < M; ++j) {
            x[j] = bits_to_float((j & 1) ? (w[j >> 1] & 0xFFFF0000u) : (w[j >> 1] << 16));
            const float a = bits_to_float(float_to_bits(x[j]) & 0x7FFFFFFFu);
            total = __fadd_rn(total, a);
            kept = ((flag[j >> 1] >> (16 * (j & 1))) & 1u) ? __fadd_rn(kept, a) : kept;
        }
        const float scale = (kept == 0.0f) ? 1.0f : __fdiv_rn(total, kept);
#pragma unroll
        for (int i = 0; i < M / 2; ++i)
            o[i] = pk_mul(float2_to_bf16x2(__fmul_rn(x[2 * i], scale), __fmul_rn(x[2 * i + 1], scale)), flag[i]);
    } else {
#pragma unroll
        for (int i = 0; i < M / 2; ++i) o[i] = pk_mul(w[i], flag[i]);
    }
}

__host__ __device__ __forceinline__ uint32_t sdgp_umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__host__ __device__ __forceinline__ uint32_t sdgp_umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
__host__ __device__ __forceinline__ uint32_t sdgp_rotl(uint32_t x, int s) { return (x << s) | (x >> (32 - s)); }
// v_perm_b32 for selector bytes 0..7 (byte i of hi:lo) and 12 (zero).
__host__ __device__ __forceinline__ uint32_t sdgp_perm(uint32_t hi, uint32_t lo, uint32_t sel) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_perm(hi, lo, sel);
#else
    const uint64_t both = ((uint64_t)hi << 32) | lo;
    uint32_t r = 0;
    for (int i = 0; i < 4; ++i) {
        const uint32_t c = (sel >> (8 * i)) & 0xFFu;
        r |= (c < 8 ? (uint32_t)((both >> (8 * c)) & 0xFFu) : 0u) << (8 * i);
    }
    return r;
#endif
}

template <int M, int RK>
__host__ __device__ __forceinline__ void prune_compress16_bf16(const uint32_t (&w)[8], int n, uint32_t (&packed)[4],
                                                               uint32_t& meta) {
    static_assert(M == 4 || M == 8 || M == 16, "group sizes that tile sixteen channels");
    static_assert(RK == kGreedy || RK == kAdjusted, "magnitude rankers only");
    constexpr uint32_t kKeyMask = 0xFFFE0001u;  // magnitude and sign
    constexpr uint32_t kCodeMask = 0x1Eu;       // what remains of a dropped key: its position
    // the mark tells a kept zero from a dropped slot, which only the rescale has to know; without it the
    // position code is an inline constant and a key costs two instructions
    constexpr uint32_t kMark = (RK == kAdjusted) ? 0x200u : 0u;
    const bool two = n >= 2;
    uint32_t f[4], s[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t d01 = w[2 * q], d23 = w[2 * q + 1];
        const uint32_t c0 = ((uint32_t)(M - 1 - (4 * q) % M) << 1) | kMark;  // code of the quad's first element
        const uint32_t k0 = (sdgp_rotl(d01, 17) & kKeyMask) | c0;
        const uint32_t k1 = (sdgp_rotl(d01, 1) & kKeyMask) | (c0 - 2u);
        const uint32_t k2 = (sdgp_rotl(d23, 17) & kKeyMask) | (c0 - 4u);
        const uint32_t k3 = (sdgp_rotl(d23, 1) & kKeyMask) | (c0 - 6u);
        const uint32_t hi = sdgp_umax(k0, k1), lo = sdgp_umin(k0, k1);
        const uint32_t hi2 = sdgp_umax(k2, k3), lo2 = sdgp_umin(k2, k3);
        f[q] = sdgp_umax(hi, hi2);
        s[q] = sdgp_umax(sdgp_umax(sdgp_umin(hi, hi2), lo), lo2);
    }
    // drop what is below the group's threshold
    if constexpr (M == 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q) s[q] = two ? s[q] : (s[q] & kCodeMask);
    } else {
#pragma unroll
        for (int g = 0; g < 16 / M; ++g) {
            constexpr int QG = M / 4;  // quads per group
            uint32_t v1 = f[g * QG], v2 = s[g * QG];
#pragma unroll
            for (int i = 1; i < QG; ++i) {
                const uint32_t fq = f[g * QG + i], sq = s[g * QG + i];
                v2 = sdgp_umax(sdgp_umax(sdgp_umin(v1, fq), v2), sq);
                v1 = sdgp_umax(v1, fq);
            }
            const uint32_t thr = two ? v2 : v1;
#pragma unroll
            for (int i = 0; i < QG; ++i) {
                const int q = g * QG + i;
                f[q] = f[q] >= thr ? f[q] : (f[q] & kCodeMask);
                s[q] = s[q] >= thr ? s[q] : (s[q] & kCodeMask);
            }
        }
    }
    float total[16 / M];
    if constexpr (RK == kAdjusted) {
#pragma unroll
        for (int g = 0; g < 16 / M; ++g) {
            float t = 0.0f;
#pragma unroll
            for (int i = 0; i < M / 2; ++i) {
                const uint32_t d = w[g * (M / 2) + i];
                t = __fadd_rn(t, bits_to_float((d << 16) & 0x7FFF0000u));
                t = __fadd_rn(t, bits_to_float(d & 0x7FFF0000u));
            }
            total[g] = t;
        }
    }
    uint32_t inv = 0;
    uint32_t lo_key[4], hi_key[4];  // rotated keys of the lower / higher position of each quad
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t ra = sdgp_rotl(f[q], 23), rb = sdgp_rotl(s[q], 23);
        const uint32_t x = sdgp_umax(ra, rb), y = sdgp_umin(ra, rb);  // the larger code is the lower position
        lo_key[q] = x, hi_key[q] = y;
#if defined(__HIP_DEVICE_COMPILE__)
        packed[q] = __builtin_amdgcn_perm(y, x, 0x06050201u);
#else
        packed[q] = ((x >> 8) & 0xFFFFu) | ((y << 8) & 0xFFFF0000u);
#endif
        inv |= (((x >> 24) & 3u) | (((y >> 24) & 3u) << 2)) << (4 * q);
    }
    meta = inv ^ 0xFFFFu;  // position = 3 - code
    if constexpr (RK == kAdjusted) {
#pragma unroll
        for (int g = 0; g < 16 / M; ++g) {
            constexpr int QG = M / 4;
            float kept = 0.0f;  // kept magnitudes in ascending position; empty slots add +0, which is exact
#pragma unroll
            for (int i = 0; i < QG; ++i) {
                const uint32_t d = packed[g * QG + i];
                kept = __fadd_rn(kept, bits_to_float((d << 16) & 0x7FFF0000u));
                kept = __fadd_rn(kept, bits_to_float(d & 0x7FFF0000u));
            }
            const float scale = (kept == 0.0f) ? 1.0f : __fdiv_rn(total[g], kept);
#pragma unroll
            for (int i = 0; i < QG; ++i) {
                const int q = g * QG + i;
                const uint32_t d = packed[q];
                const uint32_t y = float2_to_bf16x2(__fmul_rn(bits_to_float(d << 16), scale),
                                                    __fmul_rn(bits_to_float(d & 0xFFFF0000u), scale));
                // a dropped slot stays +0 whatever the scale is (the mark went away with the value)
                const uint32_t mlo = (0u - (lo_key[q] & 1u)) & 0xFFFFu, mhi = (0u - (hi_key[q] & 1u)) << 16;
                packed[q] = y & (mlo | mhi);
            }
        }
    }
}

// Random with n <= 2 on sixteen consecutive bf16 channels, into the same operand format as prune_compress16_bf16.
// Key of an element: its 28-bit hash key with (15 - position in group) in the four bits below it, so the words are
// distinct and ordered exactly like (key, lower position first): the kept set is {word >= n-th largest of the group}.
// The two largest words of a quad contain every survivor of that quad.  The values are fetched by position afterwards
// (they are not part of the key).
template <int M>
__host__ __device__ __forceinline__ void prune_compress16_random(const uint32_t (&w)[8], int n, uint32_t mix, uint64_t e0,
                                                                 uint32_t (&packed)[4], uint32_t& meta) {
    static_assert(M == 4 || M == 8 || M == 16, "group sizes that tile sixteen channels");
    const bool two = n >= 2;
    uint32_t f[4], s[4];  // largest and second largest word of each quad
    // (the sixteen elements share the high word of their index: e0 is a multiple of 16, or at least of 4 in a tensor of
    // fewer than 2^32 elements -- the callers see to it)
    const uint32_t hrow = hash_row(mix, (uint32_t)(e0 >> 32));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t e_lo = (uint32_t)e0 + (uint32_t)(4 * q);            // the quad's first element
        const uint32_t c0 = (uint32_t)(15 - (4 * q) % M);
        const uint32_t hq = hash_quad(hrow, e_lo);                         // e_lo is a multiple of 4: one word per quad
        const uint32_t k0 = hash_lane(hq, 0u) | c0;
        const uint32_t k1 = hash_lane(hq, 1u) | (c0 - 1u);
        const uint32_t k2 = hash_lane(hq, 2u) | (c0 - 2u);
        const uint32_t k3 = hash_lane(hq, 3u) | (c0 - 3u);
        const uint32_t hi = sdgp_umax(k0, k1), lo = sdgp_umin(k0, k1);
        const uint32_t hi2 = sdgp_umax(k2, k3), lo2 = sdgp_umin(k2, k3);
        f[q] = sdgp_umax(hi, hi2);
        s[q] = sdgp_umax(sdgp_umin(hi, hi2), sdgp_umax(lo, lo2));
    }
    uint32_t thr[4];  // the group's threshold, per quad
#pragma unroll
    for (int g = 0; g < 16 / M; ++g) {
        constexpr int QG = M / 4;
        // the two largest words of the group: every candidate is among its quads' two largest
        uint32_t v1 = f[g * QG], v2 = s[g * QG];
#pragma unroll
        for (int i = 1; i < QG; ++i) {
            const uint32_t cf = f[g * QG + i], cs = s[g * QG + i];   // cf > cs
            v2 = sdgp_umax(sdgp_umax(sdgp_umin(v1, cf), v2), sdgp_umin(sdgp_umax(v1, cf), cs));
            v1 = sdgp_umax(v1, cf);
        }
        const uint32_t th = two ? v2 : v1;
#pragma unroll
        for (int i = 0; i < QG; ++i) thr[g * QG + i] = th;
    }
    meta = 0;
    if (M == 4 && two) {
        // 2:4 (n is uniform over the wavefront): a quad's two largest words are its survivors, nothing else to decide
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t pf = ~f[q] & 3u, ps = ~s[q] & 3u;
            const uint32_t p_lo = sdgp_umin(pf, ps), p_hi = sdgp_umax(pf, ps);
            packed[q] = sdgp_perm(w[2 * q + 1], w[2 * q], (p_lo | (p_hi << 16)) * 0x0202u + 0x01000100u);
            meta |= (p_lo | (p_hi << 2)) << (4 * q);
        }
        return;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // the quad's survivors are among its two largest words; a slot without one keeps a (dropped) position, value +0.
        // Position in the quad from the code (15 - position in the group): its complement's low two bits.
        const uint32_t pf = ~f[q] & 3u, ps = ~s[q] & 3u;
        const uint32_t p_lo = sdgp_umin(pf, ps), p_hi = sdgp_umax(pf, ps);
        // the two values leave the quad's 64 bits by a byte permutation: bytes 2p, 2p + 1 of (d23 : d01)
        uint32_t sel = (p_lo | (p_hi << 16)) * 0x0202u + 0x01000100u;
        const bool keep_f = M == 4 ? true : f[q] >= thr[q];     // (a 4-group's threshold is its own first or second word)
        const bool keep_s = M == 4 ? two : s[q] >= thr[q];
        const bool f_first = pf < ps;
        const bool keep_lo = f_first ? keep_f : keep_s, keep_hi = f_first ? keep_s : keep_f;
        sel = keep_lo ? sel : ((sel & 0xFFFF0000u) | 0x00000C0Cu);   // selector 12 yields a zero byte
        sel = keep_hi ? sel : ((sel & 0x0000FFFFu) | 0x0C0C0000u);
        packed[q] = sdgp_perm(w[2 * q + 1], w[2 * q], sel);
        meta |= (p_lo | (p_hi << 2)) << (4 * q);
    }
}

// Two survivors (value, position) of one aligned quad, positions ascending.
// out[] holds the pruned values (zero where dropped), so a slot that has no
// survivor may point at any dropped position.
__device__ __forceinline__ void compress_quad(const bool (&k)[4], const uint32_t (&o)[4], uint32_t& v0, uint32_t& v1,
                                              uint32_t& pos) {
    const uint32_t p0 = k[0] ? 0u : (k[1] ? 1u : (k[2] ? 2u : 0u));
    v0 = k[0] ? o[0] : (k[1] ? o[1] : (k[2] ? o[2] : o[0]));
    const bool two_low = k[2] && (k[0] || k[1]);
    const bool both01 = k[1] && k[0];
    const uint32_t p1 = k[3] ? 3u : (two_low ? 2u : (both01 ? 1u : 3u));
    v1 = k[3] ? o[3] : (two_low ? o[2] : (both01 ? o[1] : o[3]));
    pos = p0 | (p1 << 2);
}

// Sixteen consecutive bf16 channels (eight dwords), n <= 2 of m in {4, 8, 16}, any ranker -> the operand format of the
// structured-sparse matrix instructions.  e0 = flat index of the first channel (Random only).
template <int M, int RK>
__device__ __forceinline__ void prune_compress16(const uint32_t (&w)[8], int n, uint32_t mix, uint64_t e0, uint32_t (&packed)[4],
                                                 uint32_t& meta) {
    if constexpr (RK != kRandom) {
        prune_compress16_bf16<M, RK>(w, n, packed, meta);
    } else {
        prune_compress16_random<M>(w, n, mix, e0, packed, meta);
    }
}

}  // namespace sdgp
