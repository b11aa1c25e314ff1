// Rescaled Magnitude with one factor per channel (Sec. III-B; the captions of the figures showing the rescaled
// gradient state that the L1 norm is preserved per channel over the batch and spatial dimensions).
//
// The kept set of every group is the Magnitude one.  Channel c of the whole tensor gets one factor
//     s[c] = (sum over rows of |dO[i,c]|) / (sum over rows that kept c of |dO[i,c]|),   1 when the divisor is 0,
// so the factor is known only after a sweep over the tensor.  Four kernels:
//   channel_sums      one streaming read of dO: ranks every group, accumulates both column sums in fp64.  A thread
//                     owns one 16-byte column slot (at least one group) and walks down the rows, so its 2 x slot
//                     accumulators live in registers; the threads of a workgroup that share a slot are added up
//                     in LDS in a fixed order, and every workgroup writes one partial sum per channel and kind
//   channel_finish    adds the partial rows in a fixed order (deterministic: no atomics) and divides
//   prune_scaled      Alg. 1 with kept values multiplied by their channel's factor (fp32 product, rounded to the
//                     storage type): same thread-to-column mapping, the factors stay in registers
//   scale_rows        W'[k,:] = W[k,:] * s[k]: folds the factors into the filter, after which the fused
//                     Magnitude backward-data kernels compute the rescaled product without a second sweep of dO
//                     (dD = sum_k x_k s_k W_k = sum_k x_k W'_k)
// All of it is bound by HBM: 2 bytes per element read for the sums, 4 for prune_scaled.
#include "ranker.h"

namespace sdgp {

namespace {

constexpr int kBlock = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One 16-byte load of a streamed tensor.  With one vector per thread the line is used up by the load and gets the
// streaming hint; with several, the lanes of one load leave gaps that the thread's other loads fill, so the line
// should stay until they have come by.
template <bool kStream>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
    if constexpr (kStream) return __builtin_nontemporal_load(p);
    else return *p;
}

template <int DT>
struct Elem;
template <>
struct Elem<kF32> {
    using type = uint32_t;
    static constexpr int kPerVec = 4;
};
template <>
struct Elem<kBF16> {
    using type = uint16_t;
    static constexpr int kPerVec = 8;
};

// How the tensor is dealt to threads.  A slot is `slot` consecutive channels (a whole number of groups); a workgroup
// is tg slots wide and tr = 256 / tg rows tall; workgroup (x, y) starts at slot x*tg and row y*tr and walks down in
// steps of nb*tr rows.
struct Plan {
    int slot;        // channels per slot
    int64_t nslots;  // C / slot
    int tg, tr;      // threads along the slots / along the rows
    int gx;          // workgroups along the slots
    int nb;          // workgroups along the rows = rows of partial sums
    bool vec;        // compiled group size and 16-byte accesses
};

// min_rows: fewest rows a thread should walk (the sums kernel writes one row of partial sums per workgroup, so its
// threads must amortise it; the pruning kernel has no such cost).
Plan make_plan(int64_t rows, int64_t C, int dt, int m, bool aligned, int min_rows, int max_wgs = 2048) {
    Plan p;
    const int pv = (dt == kBF16) ? 8 : 4;
    const int item = m > pv ? m : pv;
    p.vec = aligned && (m == 4 || m == 8 || m == 16 || m == 32) && (C % item) == 0;
    p.slot = p.vec ? item : m;
    p.nslots = C / p.slot;
    int tg = 1;
    while (tg < kBlock && tg < p.nslots) tg <<= 1;
    p.tg = tg;
    p.tr = kBlock / tg;
    p.gx = (int)((p.nslots + tg - 1) / tg);
    // about max_wgs workgroups in all; 64 rows per thread when the tensor is large enough for that many, fewer (down
    // to min_rows) when it is not
    const int64_t cap = max_wgs / p.gx > 0 ? max_wgs / p.gx : 1;
    int64_t nb = rows / ((int64_t)p.tr * 64);
    if (nb < cap) nb = rows / ((int64_t)p.tr * min_rows);
    if (nb > cap) nb = cap;
    if (nb < 1) nb = 1;
    p.nb = (int)nb;
    return p;
}

constexpr int kSumsMinRows = 16, kPruneMinRows = 2;

// The sums kernel keeps 2 x slot fp64 accumulators per thread: its workgroups should all be resident at once (a second,
// sparse round of workgroups hides no latency), which the registers of the group size bound: four workgroups of four
// wavefronts per CU up to m = 8, three at 16, two at 32.
int sums_max_wgs(int m) { return m <= 4 ? 1792 : m == 8 ? 1280 : m == 16 ? 768 : 512; }

// Keep flags of one group by Magnitude; m compiled (M > 0) or at run time (M == 0, rank count).
template <int DT, int M, bool NLE2>
__device__ __forceinline__ void magnitude_keep(const uint32_t (&raw)[M ? M : 32], int m, int n, bool (&keep)[M ? M : 32]) {
    if constexpr (M > 0) {
        uint32_t out[M];
        prune_group<DT, M, kGreedy, NLE2, false>(raw, n, 0u, 0u, keep, out);
    } else {
        constexpr uint32_t kMagMask = (DT == kBF16) ? 0x7FFFu : 0x7FFFFFFFu;
        for (int j = 0; j < m; ++j) {
            int rank = 0;
            const uint32_t kj = raw[j] & kMagMask;
            for (int i = 0; i < m; ++i) {
                const uint32_t ki = raw[i] & kMagMask;
                rank += (ki > kj || (ki == kj && i < j)) ? 1 : 0;
            }
            keep[j] = rank < n;
        }
    }
}

// Scalar path: loads the m elements of one group into raw[] (one stored bit pattern per element).
template <int DT>
__device__ __forceinline__ void load_group_scalar(const void* dO_, int64_t elem0, int m, uint32_t (&raw)[32]) {
    using T = typename Elem<DT>::type;
    const T* src = reinterpret_cast<const T*>(dO_) + elem0;
    for (int j = 0; j < m; ++j) raw[j] = (uint32_t)src[j];
}

template <int DT>
__device__ __forceinline__ float abs_as_float(uint32_t raw) {
    return (DT == kBF16) ? bits_to_float((raw & 0x7FFFu) << 16) : bits_to_float(raw & 0x7FFFFFFFu);
}

// ------------------------------------------------------------------ column sums

// Accumulation is fp64 per thread: with at most 24 significant bits per addend the sums are exact until they span
// more than 53 bits, and carrying each sum as a pair of floats (error-free additions, six fp32 operations per term)
// measured a third slower than the fp64 additions.
template <int DT, int M, bool NLE2>
__global__ void __launch_bounds__(kBlock, (DT == kBF16 && M == 4) ? 7 : 1)
channel_sums(const void* __restrict__ dO_, int64_t rows, int64_t C, int m, int n, int slot, int64_t nslots, int tg, int tr,
             double* __restrict__ partial) {
    using T = typename Elem<DT>::type;
    constexpr int PV = Elem<DT>::kPerVec;
    constexpr int SLOT = M ? (M > PV ? M : PV) : 32;  // array size; the slot itself is `slot` channels
    constexpr int GM = M ? M : 32;
    constexpr int VECS = SLOT / PV;
    __shared__ double red[kBlock];

    const int tid = threadIdx.x;
    const int sx = tid & (tg - 1), ry = tid / tg;
    const int64_t s = (int64_t)blockIdx.x * tg + sx;
    const bool active = s < nslots;
    const int64_t step = (int64_t)gridDim.y * tr;

    double tot[SLOT], kep[SLOT];
#pragma unroll
    for (int j = 0; j < SLOT; ++j) tot[j] = 0.0, kep[j] = 0.0;

    if (active) {
        int64_t r = (int64_t)blockIdx.y * tr + ry;
        if constexpr (M > 0) {
            // kDepth rows are in flight per thread: a ring of row buffers that the unrolled loop refills in place, so
            // that a row is waited for with the later requests still outstanding.  Every request inside the loop is
            // unconditional (an address past the thread's last row is replaced by that row's, and what it returns is
            // never added), which keeps the count of outstanding requests the same on every path.  The loop takes
            // whole batches of kDepth rows; the rows left in the ring are added after it.
            constexpr int kDepth = VECS == 1 ? 3 : 2;
            u32x4 ring[kDepth][VECS];
            const char* base = reinterpret_cast<const char*>(reinterpret_cast<const T*>(dO_) + s * slot);
            const int64_t row_bytes = C * (int64_t)sizeof(T);
            auto request = [&](const char* at, u32x4 (&dst)[VECS]) {
#pragma unroll
                for (int i = 0; i < VECS; ++i) dst[i] = load16<VECS == 1>(reinterpret_cast<const u32x4*>(at) + i);
            };
            auto add_row = [&](const u32x4 (&v)[VECS]) {
                if constexpr (DT == kBF16) {
                    // bf16: an element widened to fp32 is its half of the dword moved to the top, and that word with
                    // the position code in its (zero) low bits is the ranking key.  The double of a bf16 has a zero
                    // low word, so clearing the high word alone turns it into the +0 a dropped element adds.
                    uint32_t w[SLOT / 2];
#pragma unroll
                    for (int i = 0; i < VECS; ++i) {
                        w[4 * i] = v[i].x, w[4 * i + 1] = v[i].y;
                        w[4 * i + 2] = v[i].z, w[4 * i + 3] = v[i].w;
                    }
                    auto add_one = [&](int c, uint32_t fbits, uint32_t kbits) {   // |x| into tot, kept |x| (or +0) into kep
                        tot[c] += (double)__builtin_fabsf(bits_to_float(fbits));
                        kep[c] += (double)bits_to_float(kbits);
                    };
#pragma unroll
                    for (int g = 0; g < SLOT / GM; ++g) {
                        if constexpr (GM >= 16) {
                            uint32_t gw[GM / 2], km[GM / 2];
#pragma unroll
                            for (int i = 0; i < GM / 2; ++i) gw[i] = w[g * (GM / 2) + i];
                            keep_mask_packed<GM>(gw, n, km);
#pragma unroll
                            for (int i = 0; i < GM / 2; ++i) {
                                const uint32_t mag = gw[i] & 0x7FFF7FFFu, kept = mag & km[i];
                                add_one(g * GM + 2 * i, mag << 16, kept << 16);
                                add_one(g * GM + 2 * i + 1, mag & 0xFFFF0000u, kept & 0xFFFF0000u);
                            }
                        } else {
                            uint32_t f[GM], key[GM];
                            bool keep[GM];
#pragma unroll
                            for (int j = 0; j < GM; ++j) {
                                const uint32_t word = w[(g * GM + j) / 2];
                                f[j] = (j & 1) ? (word & 0xFFFF0000u) : (word << 16);
                                key[j] = (f[j] & 0x7FFF0000u) | (uint32_t)(GM - 1 - j);   // a lower position wins a tie
                            }
                            if constexpr (NLE2) select_top2_distinct<GM>(key, n, keep);
                            else if constexpr (GM == 8) select_by_sort<GM>(key, n, keep);
                            else select_by_rank<GM>(key, n, keep);
#pragma unroll
                            for (int j = 0; j < GM; ++j) {
                                const double ad = (double)__builtin_fabsf(bits_to_float(f[j]));
                                tot[g * GM + j] += ad;
                                kep[g * GM + j] += __hiloint2double(keep[j] ? __double2hiint(ad) : 0, __double2loint(ad));
                            }
                        }
                    }
                    return;
                }
                uint32_t raw[SLOT];
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
#pragma unroll
                for (int g = 0; g < SLOT / GM; ++g) {
                    uint32_t gr[GM];
                    bool keep[GM];
#pragma unroll
                    for (int j = 0; j < GM; ++j) gr[j] = raw[g * GM + j];
                    magnitude_keep<DT, M, NLE2>(gr, m, n, keep);
#pragma unroll
                    for (int j = 0; j < GM; ++j) {
                        const float a = abs_as_float<DT>(gr[j]);
                        const double ad = (double)a;
                        tot[g * GM + j] += ad;
                        kep[g * GM + j] += keep[j] ? ad : 0.0;
                    }
                }
            };
            if (r < rows) {
                // the thread's rows are r, r + step, ...: `at` walks their addresses, `end` is the last one's
                const int64_t mine = (rows - 1 - r) / step;   // index of the thread's last row
                const char* at = base + r * row_bytes;
                const char* const end = at + mine * step * row_bytes;
                const int64_t stride = step * row_bytes;
                auto clamped = [&](const char* q) { return q < end ? q : end; };
#pragma unroll
                for (int d = 0; d < kDepth; ++d) request(clamped(at + d * stride), ring[d]);
                int64_t left = mine + 1;   // rows still to add
                for (; left >= kDepth; left -= kDepth) {
#pragma unroll
                    for (int d = 0; d < kDepth; ++d) {
                        add_row(ring[d]);
                        __builtin_amdgcn_sched_barrier(0);   // the request stays here, kDepth - 1 rows of work ahead of its wait
                        request(clamped(at + (d + kDepth) * stride), ring[d]);   // after the last use: the same registers
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    at += kDepth * stride;
                }
#pragma unroll
                for (int d = 0; d < kDepth - 1; ++d) {
                    if (d < left) add_row(ring[d]);
                }
            }
        } else {
            for (; r < rows; r += step) {
                uint32_t raw[SLOT];
                load_group_scalar<DT>(dO_, r * C + s * slot, slot, raw);
                bool keep[32];
                magnitude_keep<DT, 0, false>(raw, m, n, keep);
                for (int j = 0; j < m; ++j) {
                    const float a = abs_as_float<DT>(raw[j]);
                    const double ad = (double)a;
                    tot[j] += ad;
                    kep[j] += keep[j] ? ad : 0.0;
                }
            }
        }
    }

    // Add the tr threads that share a slot, in ascending row-lane order, one accumulator at a time.
    // partial sums are stored [which][channel][workgroup row] so that the finishing pass reads a channel's run
    const int64_t nbl = gridDim.y;
    auto reduce_one = [&](int j) {
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            double v = which ? kep[j] : tot[j];
            if (tr > 1) {
                __syncthreads();
                red[tid] = v;
                __syncthreads();
                if (ry == 0) {
                    v = red[sx];
                    for (int y = 1; y < tr; ++y) v += red[y * tg + sx];
                }
            }
            if (ry == 0 && active) partial[((int64_t)which * C + s * slot + j) * nbl + blockIdx.y] = v;
        }
    };
    if constexpr (M > 0) {
        // eight accumulators per pass: every thread parks them in LDS, then each of the 8 * tg sums of the pass is
        // added by a thread of its own over the tr row lanes, in ascending order
        __shared__ double park[8][kBlock];
#pragma unroll
        for (int pass = 0; pass < 2 * SLOT / 8; ++pass) {
            if (tr > 1) __syncthreads();
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int a = pass * 8 + q;
                park[q][tid] = a < SLOT ? tot[a % SLOT] : kep[a % SLOT];
            }
            if (tr > 1) __syncthreads();
            for (int o = tid; o < 8 * tg; o += kBlock) {
                const int q = o / tg, x = o - q * tg;
                double v = park[q][x];
                for (int y = 1; y < tr; ++y) v += park[q][y * tg + x];
                const int a = pass * 8 + q, which = a / SLOT, j = a % SLOT;
                const int64_t so = (int64_t)blockIdx.x * tg + x;
                if (so < nslots) partial[((int64_t)which * C + so * slot + j) * nbl + blockIdx.y] = v;
            }
        }
    } else {
        for (int j = 0; j < slot; ++j) reduce_one(j);
    }
}

// Adds the nb partial rows and divides.  A workgroup owns kFinC channels; kFinL threads per channel each add every
// kFinL-th partial row in ascending order, then a halving tree in LDS adds the kFinL sums: a fixed order for a given
// nb, with enough independent loads in flight that the pass is not a chain of memory latencies.
constexpr int kFinC = 2, kFinL = kBlock / kFinC;

__global__ void __launch_bounds__(kBlock)
channel_finish(const double* __restrict__ partial, int nb, int64_t C, float* __restrict__ scale, double* __restrict__ sums) {
    __shared__ double red[2][kFinL][kFinC];
    const int cx = threadIdx.x % kFinC, l = threadIdx.x / kFinC;
    const int64_t c = (int64_t)blockIdx.x * kFinC + cx;
    double tot = 0.0, kep = 0.0;
    if (c < C) {
#pragma unroll 8
        for (int b = l; b < nb; b += kFinL) {
            tot += partial[c * nb + b];
            kep += partial[(C + c) * nb + b];
        }
    }
    red[0][l][cx] = tot;
    red[1][l][cx] = kep;
    __syncthreads();
    for (int half = kFinL / 2; half >= 1; half >>= 1) {
        if (l < half) {
            red[0][l][cx] += red[0][l + half][cx];
            red[1][l][cx] += red[1][l + half][cx];
        }
        __syncthreads();
    }
    if (l != 0 || c >= C) return;
    tot = red[0][0][cx];
    kep = red[1][0][cx];
    scale[c] = (kep == 0.0) ? 1.0f : (float)(tot / kep);
    if (sums) {
        sums[c] = tot;
        sums[C + c] = kep;
    }
}

// ------------------------------------------------------ prune with the factors

template <int DT, int M, bool NLE2>
__global__ void __launch_bounds__(kBlock)
prune_scaled(const void* __restrict__ dO_, int64_t rows, int64_t C, int m, int n, int slot, int64_t nslots, int tg, int tr,
             const float* __restrict__ scale, void* __restrict__ pruned_) {
    using T = typename Elem<DT>::type;
    constexpr int PV = Elem<DT>::kPerVec;
    constexpr int SLOT = M ? (M > PV ? M : PV) : 32;
    constexpr int GM = M ? M : 32;

    const int tid = threadIdx.x;
    const int sx = tid & (tg - 1), ry = tid / tg;
    const int64_t s = (int64_t)blockIdx.x * tg + sx;
    if (s >= nslots) return;
    const int64_t step = (int64_t)gridDim.y * tr;

    float sc[SLOT];
    if constexpr (M > 0) {
#pragma unroll
        for (int j = 0; j < SLOT; ++j) sc[j] = scale[s * slot + j];
    } else {
        for (int j = 0; j < slot; ++j) sc[j] = scale[s * slot + j];
    }

    int64_t r = (int64_t)blockIdx.y * tr + ry;
    if constexpr (M > 0) {
        constexpr int VECS = SLOT / PV;
        // the next row's vectors are requested before this row's are ranked (measured: faster with one and with
        // four vectors per slot, slower with two, where the row is loaded when its turn comes)
        constexpr bool kAhead = VECS != 2;
        u32x4 cur[VECS], nxt[VECS];
        const T* base = reinterpret_cast<const T*>(dO_) + s * slot;
        if (kAhead && r < rows) {
#pragma unroll
            for (int i = 0; i < VECS; ++i) cur[i] = load16<VECS == 1>(reinterpret_cast<const u32x4*>(base + r * C) + i);
        }
        for (; r < rows; r += step) {
            const int64_t rn = kAhead ? r + step : r;
            if (rn < rows) {
#pragma unroll
                for (int i = 0; i < VECS; ++i) nxt[i] = load16<VECS == 1>(reinterpret_cast<const u32x4*>(base + rn * C) + i);
            }
            if constexpr (!kAhead) {
#pragma unroll
                for (int i = 0; i < VECS; ++i) cur[i] = nxt[i];
            }
            uint32_t raw[SLOT], out[SLOT];
#pragma unroll
            for (int i = 0; i < VECS; ++i) {
                const uint32_t w[4] = {cur[i].x, cur[i].y, cur[i].z, cur[i].w};
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
#pragma unroll
            for (int g = 0; g < SLOT / GM; ++g) {
                uint32_t gr[GM];
                bool keep[GM];
#pragma unroll
                for (int j = 0; j < GM; ++j) gr[j] = raw[g * GM + j];
                magnitude_keep<DT, M, NLE2>(gr, m, n, keep);
#pragma unroll
                for (int j = 0; j < GM; ++j) {
                    const float x = (DT == kBF16) ? bf16_to_float(gr[j]) : bits_to_float(gr[j]);
                    const float y = __fmul_rn(x, sc[g * GM + j]);
                    const uint32_t yb = (DT == kBF16) ? float_to_bf16(y) : float_to_bits(y);
                    out[g * GM + j] = keep[j] ? yb : 0u;
                }
            }
            u32x4* dst = reinterpret_cast<u32x4*>(reinterpret_cast<T*>(pruned_) + r * C + s * slot);
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
#pragma unroll
            for (int i = 0; i < VECS; ++i) cur[i] = nxt[i];
        }
    } else {
        for (; r < rows; r += step) {
            const int64_t e0 = r * C + s * slot;
            uint32_t raw[SLOT];
            load_group_scalar<DT>(dO_, e0, slot, raw);
            bool keep[32];
            magnitude_keep<DT, 0, false>(raw, m, n, keep);
            T* dst = reinterpret_cast<T*>(pruned_) + e0;
            for (int j = 0; j < m; ++j) {
                const float x = (DT == kBF16) ? bf16_to_float(raw[j]) : bits_to_float(raw[j]);
                const float y = __fmul_rn(x, sc[j]);
                const uint32_t yb = (DT == kBF16) ? float_to_bf16(y) : float_to_bits(y);
                dst[j] = (T)(keep[j] ? yb : 0u);
            }
        }
    }
}

// bf16 groups of 4 or 8: the same pruned tensor from the prune pass's shape -- a thread takes four 16-byte vectors a
// workgroup apart, all of them requested before the first is ranked, and reads the eight factors of a vector's
// channels from the (cached) factor array.  vpr = vectors per row; step = kBlock % vpr.
template <int M, bool NLE2>
__global__ void __launch_bounds__(kBlock)
prune_scaled_flat(const u32x4* __restrict__ src, uint32_t nvec, uint32_t vpr, uint32_t step, int n,
                  const float* __restrict__ scale, u32x4* __restrict__ dst) {
    constexpr int K = 4;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const uint32_t v0 = blockIdx.x * (uint32_t)(kBlock * K) + threadIdx.x;
    u32x4 in[K];
#pragma unroll
    for (int u = 0; u < K; ++u) {
        const uint32_t i = v0 + (uint32_t)u * kBlock;
        if (i < nvec) in[u] = __builtin_nontemporal_load(src + i);
    }
    uint32_t col = v0 % vpr;   // this vector's place in its row; the next one is `step` further, modulo vpr
#pragma unroll
    for (int u = 0; u < K; ++u) {
        const uint32_t i = v0 + (uint32_t)u * kBlock;
        if (i >= nvec) break;
        const f32x4* f = reinterpret_cast<const f32x4*>(scale + (size_t)col * 8);
        const f32x4 f0 = f[0], f1 = f[1];
        const float sc[8] = {f0[0], f0[1], f0[2], f0[3], f1[0], f1[1], f1[2], f1[3]};
        const uint32_t w[4] = {in[u].x, in[u].y, in[u].z, in[u].w};
        uint32_t raw[8], out[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) raw[2 * k] = w[k] & 0xFFFFu, raw[2 * k + 1] = w[k] >> 16;
#pragma unroll
        for (int g = 0; g < 8 / M; ++g) {
            uint32_t gr[M];
            bool keep[M];
#pragma unroll
            for (int j = 0; j < M; ++j) gr[j] = raw[g * M + j];
            magnitude_keep<kBF16, M, NLE2>(gr, M, n, keep);
#pragma unroll
            for (int j = 0; j < M; ++j) {
                const float y = __fmul_rn(bf16_to_float(gr[j]), sc[g * M + j]);
                out[g * M + j] = keep[j] ? float_to_bf16(y) : 0u;
            }
        }
        const u32x4 pk = {out[0] | (out[1] << 16), out[2] | (out[3] << 16), out[4] | (out[5] << 16), out[6] | (out[7] << 16)};
        __builtin_nontemporal_store(pk, dst + i);
        col += step;
        col = col >= vpr ? col - vpr : col;
    }
}

// ------------------------------------------------------------ filter rows * s

// W [C_out, inner] -> W' [C_out, inner], row k multiplied by scale[k] in fp32 and rounded to the storage type.
template <int DT>
__global__ void __launch_bounds__(kBlock)
scale_rows(const void* __restrict__ W_, const float* __restrict__ scale, void* __restrict__ out_, int64_t C_out, int64_t inner) {
    using T = typename Elem<DT>::type;
    const int64_t total = C_out * inner;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const T* W = reinterpret_cast<const T*>(W_);
    T* out = reinterpret_cast<T*>(out_);
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < total; e += stride) {
        const float s = scale[e / inner];
        const uint32_t raw = (uint32_t)W[e];
        const float x = (DT == kBF16) ? bf16_to_float(raw) : bits_to_float(raw);
        const float y = __fmul_rn(x, s);
        out[e] = (T)((DT == kBF16) ? float_to_bf16(y) : float_to_bits(y));
    }
}

// --------------------------------------------------------------------- launch

template <int DT, int M>
void launch_sums(const Plan& p, const void* dO, int64_t rows, int64_t C, int m, int n, double* partial, hipStream_t st) {
    const dim3 grid((unsigned)p.gx, (unsigned)p.nb), block(kBlock);
    if (n <= 2)
        hipLaunchKernelGGL((channel_sums<DT, M, true>), grid, block, 0, st, dO, rows, C, m, n, p.slot, p.nslots, p.tg, p.tr, partial);
    else
        hipLaunchKernelGGL((channel_sums<DT, M, false>), grid, block, 0, st, dO, rows, C, m, n, p.slot, p.nslots, p.tg, p.tr, partial);
}

template <int DT, int M>
void launch_prune(const Plan& p, const void* dO, int64_t rows, int64_t C, int m, int n, const float* scale, void* pruned,
                  hipStream_t st) {
    const dim3 grid((unsigned)p.gx, (unsigned)p.nb), block(kBlock);
    if (n <= 2)
        hipLaunchKernelGGL((prune_scaled<DT, M, true>), grid, block, 0, st, dO, rows, C, m, n, p.slot, p.nslots, p.tg, p.tr, scale, pruned);
    else
        hipLaunchKernelGGL((prune_scaled<DT, M, false>), grid, block, 0, st, dO, rows, C, m, n, p.slot, p.nslots, p.tg, p.tr, scale, pruned);
}

template <int DT>
void sums_dtype(const Plan& p, const void* dO, int64_t rows, int64_t C, int m, int n, double* partial, hipStream_t st) {
    if (!p.vec) return launch_sums<DT, 0>(p, dO, rows, C, m, n, partial, st);
    switch (m) {
        case 4: return launch_sums<DT, 4>(p, dO, rows, C, m, n, partial, st);
        case 8: return launch_sums<DT, 8>(p, dO, rows, C, m, n, partial, st);
        case 16: return launch_sums<DT, 16>(p, dO, rows, C, m, n, partial, st);
        default: return launch_sums<DT, 32>(p, dO, rows, C, m, n, partial, st);
    }
}

template <int DT>
void prune_dtype(const Plan& p, const void* dO, int64_t rows, int64_t C, int m, int n, const float* scale, void* pruned,
                 hipStream_t st) {
    if (!p.vec) return launch_prune<DT, 0>(p, dO, rows, C, m, n, scale, pruned, st);
    switch (m) {
        case 4: return launch_prune<DT, 4>(p, dO, rows, C, m, n, scale, pruned, st);
        case 8: return launch_prune<DT, 8>(p, dO, rows, C, m, n, scale, pruned, st);
        case 16: return launch_prune<DT, 16>(p, dO, rows, C, m, n, scale, pruned, st);
        default: return launch_prune<DT, 32>(p, dO, rows, C, m, n, scale, pruned, st);
    }
}

}  // namespace

// Bytes of partial sums channel_scales_launch writes for these arguments (rows > 0, C > 0, C % m == 0).
size_t channel_scales_workspace(int64_t rows, int64_t C, int dt, int m) {
    const Plan p = make_plan(rows, C, dt, m, true, kSumsMinRows, sums_max_wgs(m));
    // the unaligned plan never has more partial rows than this bound: nb depends on tr = 256 / tg, and the
    // scalar plan's slots are no wider than the vector plan's, so take the larger of the two
    const Plan q = make_plan(rows, C, dt, m, false, kSumsMinRows, sums_max_wgs(m));
    const int nb = p.nb > q.nb ? p.nb : q.nb;
    return (size_t)nb * 2u * (size_t)C * sizeof(double);
}

// Validated arguments in.  scale [C] floats, sums [2*C] doubles or NULL, partial = the workspace.
int channel_scales_launch(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, float* scale, double* sums,
                          void* partial, hipStream_t stream) {
    const Plan p = make_plan(rows, C, dt, m, is_aligned16(dO), kSumsMinRows, sums_max_wgs(m));
    double* part = static_cast<double*>(partial);
    if (dt == kBF16) sums_dtype<kBF16>(p, dO, rows, C, m, n, part, stream);
    else sums_dtype<kF32>(p, dO, rows, C, m, n, part, stream);
    hipLaunchKernelGGL(channel_finish, dim3((unsigned)((C + kFinC - 1) / kFinC)), dim3(kBlock), 0, stream, part, p.nb, C,
                       scale, sums);
    return launch_status();
}

int prune_channel_rescaled_launch(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, const float* scale,
                                  void* pruned, hipStream_t stream) {
    const Plan p = make_plan(rows, C, dt, m, is_aligned16(dO) && is_aligned16(pruned), kPruneMinRows);
    const int64_t nvec = rows * (C / 8);
    if (dt == kBF16 && p.vec && (m == 4 || m == 8) && nvec < ((int64_t)1 << 31) && is_aligned16(scale)) {
        const uint32_t vpr = (uint32_t)(C / 8);
        const dim3 grid((unsigned)((nvec + kBlock * 4 - 1) / (kBlock * 4))), block(kBlock);
        const u32x4* src = static_cast<const u32x4*>(dO);
        u32x4* dst = static_cast<u32x4*>(pruned);
#define SDGP_FLAT(M_, NLE2_) \
    hipLaunchKernelGGL((prune_scaled_flat<M_, NLE2_>), grid, block, 0, stream, src, (uint32_t)nvec, vpr, (uint32_t)kBlock % vpr, n, scale, dst)
        if (m == 4) { if (n <= 2) SDGP_FLAT(4, true); else SDGP_FLAT(4, false); }
        else { if (n <= 2) SDGP_FLAT(8, true); else SDGP_FLAT(8, false); }
#undef SDGP_FLAT
        return launch_status();
    }
    if (dt == kBF16) prune_dtype<kBF16>(p, dO, rows, C, m, n, scale, pruned, stream);
    else prune_dtype<kF32>(p, dO, rows, C, m, n, scale, pruned, stream);
    return launch_status();
}

int scale_rows_launch(const void* W, const float* scale, void* out, int64_t C_out, int64_t inner, int dt, hipStream_t stream) {
    const int64_t total = C_out * inner;
    int64_t blocks = (total + kBlock - 1) / kBlock;
    if (blocks > 4096) blocks = 4096;
    if (dt == kBF16) hipLaunchKernelGGL(scale_rows<kBF16>, dim3((unsigned)blocks), dim3(kBlock), 0, stream, W, scale, out, C_out, inner);
    else hipLaunchKernelGGL(scale_rows<kF32>, dim3((unsigned)blocks), dim3(kBlock), 0, stream, W, scale, out, C_out, inner);
    return launch_status();
}

}  // namespace sdgp
