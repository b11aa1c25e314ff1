// sdgp_prune: Alg. 1 (Sec. III-A) as a streaming HIP kernel for gfx950.
//
// Because the channel count is a multiple of m, the aligned m-groups of every
// row are also the aligned m-groups of the flattened tensor, so the kernel
// walks the tensor as a 1-D array of "items": the larger of one group and one
// 16-byte vector.  A lane owns whole groups, so ranking needs no cross-lane
// traffic and no LDS; the kernel is bound by HBM (one read and one write of
// the tensor for the dense-shaped output).
//
// Two kernels:
//   prune_items    vector loads/stores, m in {4, 8, 16, 32}, any n; the
//                  selection network is chosen at compile time (see ranker.h)
//   prune_groups   one thread per group, scalar accesses, any 1 <= n <= m <= 32;
//                  used for other m, for tails and for unaligned pointers.
#include "ranker.h"

namespace sdgp {

namespace {

constexpr int kBlock = 256;
// vector kernel: items per thread -- fewer, longer-lived wavefronts with more bytes in flight each, as far as the
// registers allow (an item of a 32-group is 64 bytes of bf16; the hash keys of the random ranker cost registers too)
constexpr int items_per_thread(int m, int rk) { return m >= 32 ? 1 : (m >= 16 || rk == SDGP_RANDOM ? 2 : 4); }
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
struct Storage;
template <>
struct Storage<kF32> {
    using type = uint32_t;
    static constexpr int kPerVec = 4;  // elements in 16 bytes
};
template <>
struct Storage<kBF16> {
    using type = uint16_t;
    static constexpr int kPerVec = 8;
};

// ------------------------------------------------------------ vector kernel

template <int DT, int M, int RK, bool NLE2, bool MASKED, bool COMPACT>
__global__ void __launch_bounds__(kBlock)
prune_items(const void* __restrict__ dO_, int64_t nitems, int n, uint32_t mix, void* __restrict__ pruned_,
            void* __restrict__ vals_, uint8_t* __restrict__ idx) {
    using T = typename Storage<DT>::type;
    constexpr int PV = Storage<DT>::kPerVec;
    constexpr int ITEM = (M > PV) ? M : PV;  // elements per item
    constexpr int VECS = ITEM / PV;          // 16-byte vectors per item
    constexpr int GROUPS = ITEM / M;         // groups per item

    // kItemsPerThread items per thread, a workgroup apart (coalesced); every load is issued before the first use
    constexpr int kItemsPerThread = items_per_thread(M, RK);
    const int64_t item0 = (int64_t)blockIdx.x * (kBlock * kItemsPerThread) + threadIdx.x;
    u32x4 vin[kItemsPerThread][VECS];
#pragma unroll
    for (int u = 0; u < kItemsPerThread; ++u) {
        const int64_t it = item0 + (int64_t)u * kBlock;
        if (it < nitems) {
            const u32x4* src = reinterpret_cast<const u32x4*>(dO_) + it * VECS;
#pragma unroll
            for (int i = 0; i < VECS; ++i) {
                // an item of several vectors leaves gaps between the lanes of one load; the vectors of the other loads
                // fill them, so the cache line should stay until they have come by: no streaming hint then
                if constexpr (VECS == 1) vin[u][i] = __builtin_nontemporal_load(src + i);
                else vin[u][i] = src[i];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kItemsPerThread; ++u) {
    const int64_t item = item0 + (int64_t)u * kBlock;
    if (item >= nitems) break;
    u32x4 v[VECS];
#pragma unroll
    for (int i = 0; i < VECS; ++i) v[i] = vin[u][i];

    if constexpr (DT == kBF16 && M == 16 && NLE2 && RK != kRandom && MASKED && !COMPACT) {
        // sixteen bf16 channels, one group, at most two survivors: rank on packed keys (ranker.h) and spread the two
        // kept values of every quad back to their positions
        const uint32_t w[8] = {v[0].x, v[0].y, v[0].z, v[0].w, v[1].x, v[1].y, v[1].z, v[1].w};
        uint32_t packed[4], meta;
        prune_compress16_bf16<16, RK>(w, n, packed, meta);
        uint32_t o[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t i0 = (meta >> (4 * q)) & 3u, i1 = (meta >> (4 * q + 2)) & 3u;
            const uint64_t x = ((uint64_t)(packed[q] & 0xFFFFu) << (16 * i0)) | ((uint64_t)(packed[q] >> 16) << (16 * i1));
            o[2 * q] = (uint32_t)x, o[2 * q + 1] = (uint32_t)(x >> 32);
        }
        u32x4* dst = reinterpret_cast<u32x4*>(pruned_) + item * VECS;
        const u32x4 p0 = {o[0], o[1], o[2], o[3]}, p1 = {o[4], o[5], o[6], o[7]};
        __builtin_nontemporal_store(p0, dst);
        __builtin_nontemporal_store(p1, dst + 1);
        continue;
    }

    if constexpr (DT == kBF16 && (M == 16 || M == 32) && !NLE2 && RK != kRandom && MASKED && !COMPACT) {
        // one group of 16 or 32 bf16 channels, any n, Magnitude keys: packed 16-bit sorting network and 0/1 arithmetic
        // (ranker.h) instead of the pairwise rank count
        uint32_t w[M / 2], o[M / 2];
#pragma unroll
        for (int i = 0; i < VECS; ++i) w[4 * i] = v[i].x, w[4 * i + 1] = v[i].y, w[4 * i + 2] = v[i].z, w[4 * i + 3] = v[i].w;
        prune_packed<M, RK>(w, n, o);
        u32x4* dst = reinterpret_cast<u32x4*>(pruned_) + item * VECS;
#pragma unroll
        for (int i = 0; i < VECS; ++i) {
            const u32x4 pk = {o[4 * i], o[4 * i + 1], o[4 * i + 2], o[4 * i + 3]};
            __builtin_nontemporal_store(pk, dst + i);
        }
        continue;
    }

    uint32_t raw[ITEM];
#pragma unroll
    for (int i = 0; i < VECS; ++i) {
        const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if constexpr (DT == kBF16) {
                raw[i * 8 + 2 * k] = w[k] & 0xFFFFu;
                raw[i * 8 + 2 * k + 1] = w[k] >> 16;
            } else {
                raw[i * 4 + k] = w[k];
            }
        }
    }

    const uint64_t e0 = (uint64_t)item * ITEM;  // flat index of the item's first element
    const uint32_t hrow = hash_row(mix, (uint32_t)(e0 >> 32));

    uint32_t out[ITEM];
    bool keep[ITEM];
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        uint32_t r[M], o[M];
        bool k[M];
#pragma unroll
        for (int j = 0; j < M; ++j) r[j] = raw[g * M + j];
        prune_group<DT, M, RK, NLE2, false>(r, n, hrow, (uint32_t)e0 + g * M, k, o);
#pragma unroll
        for (int j = 0; j < M; ++j) {
            out[g * M + j] = o[j];
            keep[g * M + j] = k[j];
        }
    }

    if constexpr (MASKED) {
        u32x4* dst = reinterpret_cast<u32x4*>(pruned_) + item * VECS;
#pragma unroll
        for (int i = 0; i < VECS; ++i) {
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if constexpr (DT == kBF16) w[k] = out[i * 8 + 2 * k] | (out[i * 8 + 2 * k + 1] << 16);
                else w[k] = out[i * 4 + k];
            }
            const u32x4 pk = {w[0], w[1], w[2], w[3]};
            __builtin_nontemporal_store(pk, dst + i);
        }
    }

    if constexpr (COMPACT) {
        // Kept values and positions in ascending position; n per group.
        T* vals = reinterpret_cast<T*>(vals_);
        int64_t o = (int64_t)item * GROUPS * n;
        if (n == 2) {
            // exactly two survivors per group: the lowest and the highest kept position, found with select chains;
            // an item's values and positions leave with one store each
            uint32_t cv[GROUPS * 2], cp[GROUPS * 2];
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                uint32_t v0 = out[g * M + M - 1], p0 = M - 1, v1 = out[g * M], p1 = 0;
#pragma unroll
                for (int j = M - 2; j >= 0; --j) {
                    v0 = keep[g * M + j] ? out[g * M + j] : v0;
                    p0 = keep[g * M + j] ? (uint32_t)j : p0;
                }
#pragma unroll
                for (int j = 1; j < M; ++j) {
                    v1 = keep[g * M + j] ? out[g * M + j] : v1;
                    p1 = keep[g * M + j] ? (uint32_t)j : p1;
                }
                cv[2 * g] = v0, cv[2 * g + 1] = v1, cp[2 * g] = p0, cp[2 * g + 1] = p1;
            }
            if constexpr (DT == kBF16 && GROUPS == 2) {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 pv = {cv[0] | (cv[1] << 16), cv[2] | (cv[3] << 16)};
                __builtin_nontemporal_store(pv, reinterpret_cast<u32x2*>(vals + o));
                __builtin_nontemporal_store(cp[0] | (cp[1] << 8) | (cp[2] << 16) | (cp[3] << 24), reinterpret_cast<uint32_t*>(idx + o));
            } else if constexpr (DT == kBF16) {
                static_assert(GROUPS == 1, "one group per item");
                __builtin_nontemporal_store(cv[0] | (cv[1] << 16), reinterpret_cast<uint32_t*>(vals + o));
                __builtin_nontemporal_store((uint16_t)(cp[0] | (cp[1] << 8)), reinterpret_cast<uint16_t*>(idx + o));
            } else {
                static_assert(GROUPS == 1, "one group per item");
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 pv = {cv[0], cv[1]};
                __builtin_nontemporal_store(pv, reinterpret_cast<u32x2*>(vals + o));
                __builtin_nontemporal_store((uint16_t)(cp[0] | (cp[1] << 8)), reinterpret_cast<uint16_t*>(idx + o));
            }
            continue;
        }
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
#pragma unroll
            for (int j = 0; j < M; ++j) {
                if (keep[g * M + j]) {
                    vals[o] = (T)out[g * M + j];
                    idx[o] = (uint8_t)j;
                    ++o;
                }
            }
        }
    }
    }  // items of this thread
}

// ----------------------------------------------- 16- and 32-channel groups of bf16, dense-shaped output
//
// One lane per group means 32 or 64 bytes per lane, and a wavefront's 16-byte loads and stores then touch every
// second or fourth 16 bytes of the span it covers: measured at 3 TB/s for 64 bytes per lane even when the ranking is a
// handful of instructions (2:32).  Here a wavefront moves its 2 or 4 KB with whole-line accesses (lane i takes vector
// i of each 1 KB part) and the vectors change lanes through LDS on the way in and on the way out; slot c of a
// wavefront's region holds vector c ^ ((c >> 4) & (V - 1)), V vectors per group, which keeps both the row-wise and
// the group-wise accesses free of bank conflicts.
// A wavefront's LDS writes before this point are visible to its own lanes' reads after it (the regions below belong to
// one wavefront each, so no workgroup barrier is needed: the LDS serves a wavefront's instructions in order).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int M, int RK, bool NLE2>
__global__ void __launch_bounds__(kBlock)
prune_items_wide(const void* __restrict__ dO_, int64_t nitems, int n, uint32_t mix, void* __restrict__ pruned_) {
    static_assert(M == 16 || M == 32, "two or four vectors per group");
    constexpr int V = M / 8;
    __shared__ u32x4 stage[kBlock * V];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t item = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t vec0 = ((int64_t)blockIdx.x * kBlock + wave * 64) * V;   // first vector of this wavefront's 64 groups
    const int64_t nvec = nitems * V;
    u32x4* region = stage + wave * (64 * V);
    const u32x4* src = reinterpret_cast<const u32x4*>(dO_);
    u32x4 in[V];
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const int c = k * 64 + lane;
        in[k] = u32x4{0u, 0u, 0u, 0u};
        if (vec0 + c < nvec) in[k] = __builtin_nontemporal_load(src + vec0 + c);
    }
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const int c = k * 64 + lane;
        region[c ^ ((c >> 4) & (V - 1))] = in[k];
    }
    wave_lds_sync();
    uint32_t w[M / 2];
#pragma unroll
    for (int p = 0; p < V; ++p) {
        const int c = V * lane + p;
        const u32x4 v = region[c ^ ((c >> 4) & (V - 1))];
        w[4 * p] = v.x, w[4 * p + 1] = v.y, w[4 * p + 2] = v.z, w[4 * p + 3] = v.w;
    }
    uint32_t o[M / 2];
    if constexpr (!NLE2 && RK != kRandom) {
        prune_packed<M, RK>(w, n, o);
    } else {
        uint32_t r[M], out[M];
        bool keep[M];
#pragma unroll
        for (int i = 0; i < M / 2; ++i) r[2 * i] = w[i] & 0xFFFFu, r[2 * i + 1] = w[i] >> 16;
        const uint64_t e0 = (uint64_t)item * M;   // (a group past the end is ranked on zeros and never stored)
        prune_group<kBF16, M, RK, NLE2, false>(r, n, hash_row(mix, (uint32_t)(e0 >> 32)), (uint32_t)e0, keep, out);
#pragma unroll
        for (int i = 0; i < M / 2; ++i) o[i] = out[2 * i] | (out[2 * i + 1] << 16);
    }
    wave_lds_sync();   // every lane has read its group
#pragma unroll
    for (int p = 0; p < V; ++p) {
        const int c = V * lane + p;
        region[c ^ ((c >> 4) & (V - 1))] = u32x4{o[4 * p], o[4 * p + 1], o[4 * p + 2], o[4 * p + 3]};
    }
    wave_lds_sync();
    u32x4* dst = reinterpret_cast<u32x4*>(pruned_);
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const int c = k * 64 + lane;
        if (vec0 + c < nvec) __builtin_nontemporal_store(region[c ^ ((c >> 4) & (V - 1))], dst + vec0 + c);
    }
}

// ------------------------------------------------------------- group kernel

template <int DT>
__global__ void __launch_bounds__(kBlock)
prune_groups(const void* __restrict__ dO_, int64_t ngroups, int64_t e_base, int n, int m, int rk, uint32_t mix,
             void* __restrict__ pruned_, void* __restrict__ vals_, uint8_t* __restrict__ idx) {
    using T = typename Storage<DT>::type;
    const int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (g >= ngroups) return;
    const T* src = reinterpret_cast<const T*>(dO_) + g * m;
    constexpr uint32_t kMagMask = (DT == kBF16) ? 0x7FFFu : 0x7FFFFFFFu;

    uint32_t raw[32], key[32];
    const uint64_t e0 = (uint64_t)e_base + (uint64_t)g * (uint64_t)m;
    for (int j = 0; j < m; ++j) {
        raw[j] = (uint32_t)src[j];
        const uint64_t e = e0 + (uint64_t)j;
        key[j] = (rk == kRandom) ? hash_elem(hash_row(mix, (uint32_t)(e >> 32)), (uint32_t)e) : (raw[j] & kMagMask);
    }
    uint32_t keepmask = 0;
    for (int j = 0; j < m; ++j) {
        int rank = 0;
        for (int i = 0; i < m; ++i) rank += (key[i] > key[j] || (key[i] == key[j] && i < j)) ? 1 : 0;
        if (rank < n) keepmask |= 1u << j;
    }
    float scale = 1.0f;
    if (rk == kAdjusted) {
        float total = 0.0f, kept = 0.0f;
        for (int j = 0; j < m; ++j) {
            const float x = (DT == kBF16) ? bf16_to_float(raw[j]) : bits_to_float(raw[j]);
            const float a = bits_to_float(float_to_bits(x) & 0x7FFFFFFFu);
            total = __fadd_rn(total, a);
            if ((keepmask >> j) & 1u) kept = __fadd_rn(kept, a);
        }
        scale = (kept == 0.0f) ? 1.0f : __fdiv_rn(total, kept);
    }
    T* pruned = reinterpret_cast<T*>(pruned_);
    T* vals = reinterpret_cast<T*>(vals_);
    int64_t o = g * n;
    for (int j = 0; j < m; ++j) {
        uint32_t y = 0;
        const bool k = (keepmask >> j) & 1u;
        if (k) {
            y = raw[j];
            if (rk == kAdjusted) {
                const float x = (DT == kBF16) ? bf16_to_float(raw[j]) : bits_to_float(raw[j]);
                const float p = __fmul_rn(x, scale);
                y = (DT == kBF16) ? float_to_bf16(p) : float_to_bits(p);
            }
        }
        if (pruned) pruned[g * m + j] = (T)y;
        if (k && vals) {
            vals[o] = (T)y;
            idx[o] = (uint8_t)j;
            ++o;
        }
    }
}

// ------------------------------------------------------------------ dispatch

struct PruneArgs {
    const void* dO;
    int64_t total;  // elements
    int n, m, rk;
    uint32_t mix;
    void* pruned;
    void* vals;
    uint8_t* idx;
    hipStream_t stream;
};

template <int DT, int M, int RK, bool NLE2>
void launch_items_out(const PruneArgs& a, int64_t nitems) {
    const int64_t per_block = (int64_t)kBlock * items_per_thread(M, RK);
    const dim3 grid((unsigned)((nitems + per_block - 1) / per_block)), block(kBlock);
    if constexpr (DT == kBF16 && (M == 16 || M == 32)) {
        if (a.pruned && !a.vals) {   // one group per thread
            const dim3 wide((unsigned)((nitems + kBlock - 1) / kBlock));
            hipLaunchKernelGGL((prune_items_wide<M, RK, NLE2>), wide, block, 0, a.stream, a.dO, nitems, a.n, a.mix, a.pruned);
            return;
        }
    }
    if (a.pruned && a.vals)
        hipLaunchKernelGGL((prune_items<DT, M, RK, NLE2, true, true>), grid, block, 0, a.stream, a.dO, nitems, a.n, a.mix,
                           a.pruned, a.vals, a.idx);
    else if (a.pruned)
        hipLaunchKernelGGL((prune_items<DT, M, RK, NLE2, true, false>), grid, block, 0, a.stream, a.dO, nitems, a.n, a.mix,
                           a.pruned, a.vals, a.idx);
    else
        hipLaunchKernelGGL((prune_items<DT, M, RK, NLE2, false, true>), grid, block, 0, a.stream, a.dO, nitems, a.n, a.mix,
                           a.pruned, a.vals, a.idx);
}

template <int DT, int M>
void launch_items(const PruneArgs& a, int64_t nitems) {
    const bool nle2 = a.n <= 2;
    switch (a.rk) {
        case kRandom:
            nle2 ? launch_items_out<DT, M, kRandom, true>(a, nitems) : launch_items_out<DT, M, kRandom, false>(a, nitems);
            break;
        case kGreedy:
            nle2 ? launch_items_out<DT, M, kGreedy, true>(a, nitems) : launch_items_out<DT, M, kGreedy, false>(a, nitems);
            break;
        default:
            nle2 ? launch_items_out<DT, M, kAdjusted, true>(a, nitems) : launch_items_out<DT, M, kAdjusted, false>(a, nitems);
            break;
    }
}

template <int DT>
void launch_groups(const PruneArgs& a, int64_t first_elem, int64_t nelems) {
    using T = typename Storage<DT>::type;
    const int64_t ngroups = nelems / a.m;
    if (ngroups == 0) return;
    const int64_t kept0 = first_elem / a.m * a.n;
    const dim3 grid((unsigned)((ngroups + kBlock - 1) / kBlock)), block(kBlock);
    hipLaunchKernelGGL((prune_groups<DT>), grid, block, 0, a.stream,
                       (const void*)(reinterpret_cast<const T*>(a.dO) + first_elem), ngroups, first_elem, a.n, a.m, a.rk,
                       a.mix, a.pruned ? (void*)(reinterpret_cast<T*>(a.pruned) + first_elem) : nullptr,
                       a.vals ? (void*)(reinterpret_cast<T*>(a.vals) + kept0) : nullptr, a.idx ? a.idx + kept0 : nullptr);
}

template <int DT>
void prune_dtype(const PruneArgs& a) {
    constexpr int PV = Storage<DT>::kPerVec;
    const bool vec_m = (a.m == 4 || a.m == 8 || a.m == 16 || a.m == 32);
    const bool aligned = is_aligned16(a.dO) && (!a.pruned || is_aligned16(a.pruned)) &&
                         (!a.vals || (is_aligned16(a.vals) && (reinterpret_cast<uintptr_t>(a.idx) & 3u) == 0));  // vector stores of the compact output
    int64_t done = 0;
    if (vec_m && aligned) {
        const int item = a.m > PV ? a.m : PV;
        const int64_t nitems = a.total / item;
        if (nitems > 0) {
            switch (a.m) {
                case 4: launch_items<DT, 4>(a, nitems); break;
                case 8: launch_items<DT, 8>(a, nitems); break;
                case 16: launch_items<DT, 16>(a, nitems); break;
                default: launch_items<DT, 32>(a, nitems); break;
            }
        }
        done = nitems * item;
    }
    if (done < a.total) launch_groups<DT>(a, done, a.total - done);
}

}  // namespace

// Validated arguments in; launches on `stream`.  total = rows * C.
int prune_launch(const void* dO, int64_t total, int dt, int n, int m, int rk, uint64_t seed, void* pruned, void* vals,
                 uint8_t* idx, hipStream_t stream) {
    PruneArgs a{dO, total, n, m, rk, seed_mix(seed), pruned, vals, idx, stream};
    if (dt == kBF16) prune_dtype<kBF16>(a);
    else prune_dtype<kF32>(a);
    return launch_status();
}

}  // namespace sdgp
