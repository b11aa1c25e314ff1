/*
 * sdgp_oracle.c -- plain CPU reference of the SDGP backward-data path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * checked against.  It shares no code with the GPU library, includes no HIP
 * header, and nothing in the product may call it: only the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg do.
 *
 * What it computes (arXiv 2202.00774):
 *   - Alg. 1 (Sec. III-A): walk over the aligned groups of m consecutive
 *     channels of dL/dO, apply the pruning function P to each, store the result
 *     at the same place of a zero-initialised copy.
 *   - the three P of Sec. III-B: Random, Magnitude ("greedy"), Rescaled
 *     Magnitude ("greedy-adjusted"), and the second reading of the latter with
 *     one factor per channel;
 *   - the backward-data product that consumes the pruned tensor (Fig. 1, Fig. 2,
 *     Fig. 3): a matrix product for a linear layer, the transposed correlation
 *     for a convolution layer;
 *   - the two other products of a layer's training step (Sec. II-A, Fig. 1): the
 *     forward convolution and the weight gradient, which takes the unpruned
 *     dL/dO (Sec. III-A).
 *
 * Arithmetic.  Ranking is integer work on bit patterns and is exact.  The
 * rescale of Rescaled Magnitude is done in IEEE fp32 in a fixed order because
 * its rounded result is compared bit for bit; this file must be compiled
 * without fast-math and without fused multiply-add contraction.  The products
 * accumulate in fp64 in the order taps -> channels.
 *
 * Readings of points the paper leaves open are marked "Reading:".
 *
 * Parity pins: every function below is pinned by tests that do not call it to
 * produce their expectation (worked example of Sec. III-B, brute-force
 * enumeration of keep-sets, closed forms, library special cases, adjoint
 * identity).  The counter hash is a definition of this build (the paper gives
 * no generator); it is pinned by stored vectors and by statistical properties.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_F32 = 0, REF_BF16 = 1 };
enum { REF_RANDOM = 0, REF_GREEDY = 1, REF_GREEDY_ADJUSTED = 2 };

/* ---------------------------------------------------------------- scalars */

static float bits_to_float(uint32_t u) {
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint32_t float_to_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return u;
}

/* bfloat16 is the upper half of a binary32. */
static float bf16_to_float(uint16_t h) { return bits_to_float((uint32_t)h << 16); }

/* binary32 -> bfloat16, round to nearest, ties to even. */
static uint16_t float_to_bf16(float f) {
    uint32_t u = float_to_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

uint16_t sdgp_ref_float_to_bf16(float f) { return float_to_bf16(f); }
float sdgp_ref_bf16_to_float(uint16_t h) { return bf16_to_float(h); }

/*
 * Counter hash for the Random ranker.  Reading: the paper only says that m-n
 * elements are pruned at random (Sec. III-B); to make the result a pure function
 * of (seed, element) the key of element e is H(seed, e) below, all arithmetic
 * modulo 2^32.  One mixed word is made per aligned quad of flat element indices
 * (e >> 2); its four elements take the four byte rotations of that word, so the
 * order of their keys is the order of four different bytes of one well mixed
 * word.  The low four bits of a key are cleared: a key is 28 bits wide, and keys
 * that agree in them tie (the lower position then wins, like any tie), which
 * leaves a kernel room to carry a position code below the key.  Constants: floor(2^32/phi) and the fractional parts of sqrt(2), sqrt(3),
 * sqrt(7), sqrt(11) scaled by 2^32.
 */
uint32_t sdgp_ref_hash(uint64_t seed, uint64_t e) {
    uint32_t x = (uint32_t)e, y = (uint32_t)(e >> 32);
    uint32_t s0 = (uint32_t)seed, s1 = (uint32_t)(seed >> 32);
    uint32_t v = 0xA54FF53Au ^ (x >> 2) ^ (s0 * 0x9E3779B9u) ^ (y * 0xBB67AE85u) ^ (s1 * 0x510E527Fu);
    v ^= v >> 16;
    v *= 0x6A09E667u;
    v ^= v >> 15;
    v *= 0xBB67AE85u;
    v ^= v >> 16;
    unsigned rot = 8u * (x & 3u);
    v = rot ? (v << rot) | (v >> (32u - rot)) : v;
    return v & 0xFFFFFFF0u;
}

/* ------------------------------------------------------------ one group */

/*
 * P(group, n) of Sec. III-B for one group of m elements.
 *   x[j]      the group's values widened to fp32 (exact for both dtypes)
 *   mag[j]    sign-cleared bit pattern of the stored value (the magnitude key)
 *   e0        flat index of the group's first element (for the hash)
 * Output: keep[j] in {0,1} with exactly n ones, scale (1 unless adjusted).
 *
 * Sec. III-B ranks the group by magnitude and keeps the top n, remembering the
 * original positions.  Reading: equal keys are ordered by position, lower
 * first; so the kept set is unique.  A group with fewer than n nonzeros still
 * keeps n positions.
 */
static void rank_group(const float* x, const uint32_t* mag, int m, int n, int ranker, uint64_t seed,
                       uint64_t e0, unsigned char* keep, float* scale) {
    uint32_t key[32];
    for (int j = 0; j < m; ++j) {
        key[j] = (ranker == REF_RANDOM) ? sdgp_ref_hash(seed, e0 + (uint64_t)j) : mag[j];
        keep[j] = 0;
    }
    for (int t = 0; t < n; ++t) {
        int best = -1;
        for (int j = 0; j < m; ++j) {
            if (keep[j]) continue;
            if (best < 0 || key[j] > key[best]) best = j; /* strict: ties stay with the lower j */
        }
        keep[best] = 1;
    }
    *scale = 1.0f;
    if (ranker == REF_GREEDY_ADJUSTED) {
        /* Rescaled Magnitude: make the L1 norm of the pruned group equal to that
         * of the group.  Reading: the norm is taken over the group P receives
         * (Alg. 1 hands P one group).  fp32, ascending order, one division. */
        float total = 0.0f, kept = 0.0f;
        for (int j = 0; j < m; ++j) {
            float a = bits_to_float(float_to_bits(x[j]) & 0x7FFFFFFFu);
            total = total + a;
            if (keep[j]) kept = kept + a;
        }
        *scale = (kept == 0.0f) ? 1.0f : total / kept;
    }
}

/* --------------------------------------------------------------- Alg. 1 */

/*
 * dO [rows, C] -> pruned [rows, C] (may be NULL), vals [rows, C*n/m] and
 * idx [rows, C*n/m] (both may be NULL).  Returns 0, or -1 on bad arguments.
 */
int sdgp_ref_prune(const void* dO, int64_t rows, int64_t C, int dtype, int n, int m, int ranker,
                   uint64_t seed, void* pruned, void* vals, uint8_t* idx) {
    if (n < 1 || n > m || m > 32 || C < 0 || rows < 0 || (C % m) != 0) return -1;
    if (dtype != REF_F32 && dtype != REF_BF16) return -1;
    if (ranker < REF_RANDOM || ranker > REF_GREEDY_ADJUSTED) return -1;
    const int64_t groups = C / m;
    const int64_t Ck = groups * n;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t g = 0; g < groups; ++g) {
            const int64_t base = i * C + g * m;
            float x[32];
            uint32_t mag[32];
            unsigned char keep[32];
            float scale;
            for (int j = 0; j < m; ++j) {
                if (dtype == REF_BF16) {
                    uint16_t h = ((const uint16_t*)dO)[base + j];
                    x[j] = bf16_to_float(h);
                    mag[j] = (uint32_t)(h & 0x7FFFu);
                } else {
                    uint32_t u = ((const uint32_t*)dO)[base + j];
                    x[j] = bits_to_float(u);
                    mag[j] = u & 0x7FFFFFFFu;
                }
            }
            rank_group(x, mag, m, n, ranker, seed, (uint64_t)base, keep, &scale);
            int t = 0;
            for (int j = 0; j < m; ++j) {
                /* kept value: a bit copy, or the rescaled value rounded to dtype */
                uint32_t out32 = 0;
                uint16_t out16 = 0;
                if (keep[j]) {
                    if (ranker == REF_GREEDY_ADJUSTED) {
                        float y = x[j] * scale;
                        out32 = float_to_bits(y);
                        out16 = float_to_bf16(y);
                    } else if (dtype == REF_BF16) {
                        out16 = ((const uint16_t*)dO)[base + j];
                    } else {
                        out32 = ((const uint32_t*)dO)[base + j];
                    }
                }
                if (pruned) {
                    if (dtype == REF_BF16) ((uint16_t*)pruned)[base + j] = out16;
                    else ((uint32_t*)pruned)[base + j] = out32;
                }
                if (keep[j]) {
                    const int64_t o = i * Ck + g * n + t;
                    if (vals) {
                        if (dtype == REF_BF16) ((uint16_t*)vals)[o] = out16;
                        else ((uint32_t*)vals)[o] = out32;
                    }
                    if (idx) idx[o] = (uint8_t)j;
                    ++t;
                }
            }
        }
    }
    return 0;
}

/* ------------------------------------- Rescaled Magnitude, per-channel norm */

/*
 * The captions of the figures that show the rescaled gradient (Sec. III-B) speak
 * of an L1 norm preserved per channel across the batch and spatial dimensions,
 * while Alg. 1 hands P one group.  Reading (the second one; the per-group reading
 * above stays the default): the kept set is the Magnitude one, and channel c gets
 * ONE factor for the whole tensor,
 *     s[c] = (sum over rows of |dO[i,c]|) / (sum over rows where c was kept of |dO[i,c]|),
 * so that the column's L1 norm after pruning equals the one before.  A column whose
 * kept sum is zero (nothing but zeros survived) has s[c] = 1.
 *
 * Arithmetic: the two column sums in fp64, rows ascending; s[c] is their fp64
 * quotient rounded once to fp32; a kept value is fp32(x) * s[c] in fp32, rounded to
 * the storage type (round to nearest even).
 *
 * Outputs (each may be NULL): total[C] and kept[C] (the fp64 sums), scale[C],
 * pruned [rows, C].  Returns 0, or -1 on bad arguments or out of memory.
 */
int sdgp_ref_prune_channel_rescaled(const void* dO, int64_t rows, int64_t C, int dtype, int n, int m,
                                    double* total, double* kept, float* scale, void* pruned) {
    if (n < 1 || n > m || m > 32 || C < 0 || rows < 0 || (C % m) != 0) return -1;
    if (dtype != REF_F32 && dtype != REF_BF16) return -1;
    const int64_t groups = C / m;
    double* tot = (double*)calloc((size_t)(C > 0 ? C : 1), sizeof(double));
    double* kep = (double*)calloc((size_t)(C > 0 ? C : 1), sizeof(double));
    float* sc = (float*)malloc((size_t)(C > 0 ? C : 1) * sizeof(float));
    unsigned char* mask = (unsigned char*)malloc((size_t)(rows * C > 0 ? rows * C : 1));
    if (!tot || !kep || !sc || !mask) {
        free(tot), free(kep), free(sc), free(mask);
        return -1;
    }
    /* first sweep: Magnitude keep-set of every group, and the two sums of every column */
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t g = 0; g < groups; ++g) {
            const int64_t base = i * C + g * m;
            float x[32], unused;
            uint32_t mag[32];
            for (int j = 0; j < m; ++j) {
                if (dtype == REF_BF16) {
                    uint16_t h = ((const uint16_t*)dO)[base + j];
                    x[j] = bf16_to_float(h);
                    mag[j] = (uint32_t)(h & 0x7FFFu);
                } else {
                    uint32_t u = ((const uint32_t*)dO)[base + j];
                    x[j] = bits_to_float(u);
                    mag[j] = u & 0x7FFFFFFFu;
                }
            }
            rank_group(x, mag, m, n, REF_GREEDY, 0, 0, mask + base, &unused);
            for (int j = 0; j < m; ++j) {
                double a = (double)bits_to_float(float_to_bits(x[j]) & 0x7FFFFFFFu);
                tot[g * m + j] += a;
                if (mask[base + j]) kep[g * m + j] += a;
            }
        }
    }
    for (int64_t c = 0; c < C; ++c) sc[c] = (kep[c] == 0.0) ? 1.0f : (float)(tot[c] / kep[c]);
    /* second sweep: kept values times their column's factor */
    if (pruned) {
        for (int64_t i = 0; i < rows; ++i) {
            for (int64_t c = 0; c < C; ++c) {
                const int64_t e = i * C + c;
                if (dtype == REF_BF16) {
                    float y = bf16_to_float(((const uint16_t*)dO)[e]) * sc[c];
                    ((uint16_t*)pruned)[e] = mask[e] ? float_to_bf16(y) : (uint16_t)0;
                } else {
                    float y = ((const float*)dO)[e] * sc[c];
                    ((uint32_t*)pruned)[e] = mask[e] ? float_to_bits(y) : 0u;
                }
            }
        }
    }
    if (total) memcpy(total, tot, (size_t)C * sizeof(double));
    if (kept) memcpy(kept, kep, (size_t)C * sizeof(double));
    if (scale) memcpy(scale, sc, (size_t)C * sizeof(float));
    free(tot), free(kep), free(sc), free(mask);
    return 0;
}

/* ------------------------------------------------------ backward products */

static double load_as_double(const void* p, int64_t i, int dtype) {
    if (dtype == REF_BF16) return (double)bf16_to_float(((const uint16_t*)p)[i]);
    return (double)((const float*)p)[i];
}

/*
 * Linear layer (Fig. 2 right): dD[i,c] = sum_k dOp[i,k] * W[k,c], with dOp the
 * (already pruned, dense-shaped) output gradient [rows, C_out] and W [C_out, C_in].
 * Also returns absum[i,c] = sum_k |dOp[i,k]| * |W[k,c]|, the scale against which
 * a rounding error of the product is judged.  fp64 accumulation, k ascending.
 */
int sdgp_ref_linear_bwd_data(const void* dOp, const void* W, int64_t rows, int64_t C_out, int64_t C_in,
                             int dtype, double* dD, double* absum) {
    if (rows < 0 || C_out < 0 || C_in < 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t c = 0; c < C_in; ++c) {
            double acc = 0.0, mag = 0.0;
            for (int64_t k = 0; k < C_out; ++k) {
                double a = load_as_double(dOp, i * C_out + k, dtype);
                double w = load_as_double(W, k * C_in + c, dtype);
                acc += a * w;
                mag += (a < 0 ? -a : a) * (w < 0 ? -w : w);
            }
            dD[i * C_in + c] = acc;
            if (absum) absum[i * C_in + c] = mag;
        }
    }
    return 0;
}

/* One input pixel of the convolution backward-data (see below). */
static void conv_pixel(const void* dOp, const void* W, int64_t b, int64_t h, int64_t w, int64_t P,
                       int64_t Q, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad,
                       int dtype, double* out, double* mag) {
    for (int64_t c = 0; c < C_in; ++c) {
        double acc = 0.0, am = 0.0;
        for (int r = 0; r < R; ++r) {
            int64_t hp = h + pad - r;
            if (hp < 0 || hp % stride != 0) continue;
            int64_t p = hp / stride;
            if (p >= P) continue;
            for (int s = 0; s < S; ++s) {
                int64_t wq = w + pad - s;
                if (wq < 0 || wq % stride != 0) continue;
                int64_t q = wq / stride;
                if (q >= Q) continue;
                for (int64_t k = 0; k < C_out; ++k) {
                    double a = load_as_double(dOp, ((b * P + p) * Q + q) * C_out + k, dtype);
                    double v = load_as_double(W, ((k * R + r) * S + s) * C_in + c, dtype);
                    acc += a * v;
                    am += (a < 0 ? -a : a) * (v < 0 ? -v : v);
                }
            }
        }
        out[c] = acc;
        if (mag) mag[c] = am;
    }
}

/*
 * Convolution layer (Fig. 3 left).  The forward pass was the cross-correlation
 *   O[b,p,q,k] = sum_{r,s,c} D[b, p*stride + r - pad, q*stride + s - pad, c] * W[k,r,s,c]
 * (Reading: correlation, dilation 1, one group, weights stored [C_out,R,S,C_in]).
 * Differentiating with respect to D gives
 *   dD[b,h,w,c] = sum_{r,s} sum_k dOp[b,p,q,k] * W[k,r,s,c]
 * over the taps for which p = (h+pad-r)/stride and q = (w+pad-s)/stride are
 * integers inside the output.  dOp [B,P,Q,C_out] is the pruned tensor; dD and
 * absum are [B,H,Wd,C_in] in fp64.
 */
int sdgp_ref_conv_bwd_data(const void* dOp, const void* W, int64_t B, int64_t H, int64_t Wd,
                           int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dtype,
                           double* dD, double* absum) {
    if (B < 0 || H < 0 || Wd < 0 || C_in < 0 || C_out < 0 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return -1;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return -1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    const int64_t npix = B * H * Wd;
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < npix; ++pix) {
        int64_t w = pix % Wd, h = (pix / Wd) % H, b = pix / (Wd * H);
        conv_pixel(dOp, W, b, h, w, P, Q, C_in, C_out, R, S, stride, pad, dtype, dD + pix * C_in,
                   absum ? absum + pix * C_in : NULL);
    }
    return 0;
}

/*
 * The same sum for a chosen list of input pixels: pixels[t] is the flat index
 * (b*H + h)*Wd + w; dD and absum are [count, C_in].  Used to check full-size
 * tensors at sampled positions.
 */
int sdgp_ref_conv_bwd_data_at(const void* dOp, const void* W, int64_t B, int64_t H, int64_t Wd,
                              int64_t C_in, int64_t C_out, int R, int S, int stride, int pad,
                              int dtype, const int64_t* pixels, int64_t count, double* dD,
                              double* absum) {
    if (B < 0 || H < 0 || Wd < 0 || C_in < 0 || C_out < 0 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return -1;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return -1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    for (int64_t t = 0; t < count; ++t)
        if (pixels[t] < 0 || pixels[t] >= B * H * Wd) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t) {
        int64_t pix = pixels[t];
        int64_t w = pix % Wd, h = (pix / Wd) % H, b = pix / (Wd * H);
        conv_pixel(dOp, W, b, h, w, P, Q, C_in, C_out, R, S, stride, pad, dtype, dD + t * C_in,
                   absum ? absum + t * C_in : NULL);
    }
    return 0;
}

/*
 * Grouped convolution (the RegNetX layers of Sec. IV): the channels are split into `groups` independent convolutions.
 * Output channel k belongs to group g = k / (C_out/groups) and sees only the input channels
 * [g*C_in/groups, (g+1)*C_in/groups); W is [C_out, R, S, C_in/groups].  Differentiating
 *   O[b,p,q,k] = sum_{r,s} sum_{c' < C_in/groups} D[b, p*stride+r-pad, q*stride+s-pad, g*C_in/groups + c'] * W[k,r,s,c']
 * with respect to D: input channel c of group g = c / (C_in/groups) collects the output channels of its group only,
 *   dD[b,h,w,c] = sum_{r,s} sum_{k in group g} dOp[b,p,q,k] * W[k,r,s, c - g*C_in/groups].
 * dOp is the pruned tensor (pruned along all of C_out as one row: Alg. 1 does not know about groups).  With
 * pixels != NULL only the input pixels pixels[t] = (b*H + h)*Wd + w are computed, as [count, C_in].
 */
int sdgp_ref_conv_bwd_data_grouped(const void* dOp, const void* W, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                                   int64_t C_out, int R, int S, int stride, int pad, int64_t groups, int dtype,
                                   const int64_t* pixels, int64_t count, double* dD, double* absum) {
    if (B < 0 || H < 0 || Wd < 0 || C_in < 0 || C_out < 0 || R < 1 || S < 1 || stride < 1 || pad < 0) return -1;
    if (groups < 1 || C_in % groups != 0 || C_out % groups != 0) return -1;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return -1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    const int64_t cig = C_in / groups, cog = C_out / groups;
    const int64_t npix = pixels ? count : B * H * Wd;
    for (int64_t t = 0; pixels && t < count; ++t)
        if (pixels[t] < 0 || pixels[t] >= B * H * Wd) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < npix; ++t) {
        const int64_t pix = pixels ? pixels[t] : t;
        const int64_t w = pix % Wd, h = (pix / Wd) % H, b = pix / (Wd * H);
        for (int64_t c = 0; c < C_in; ++c) {
            const int64_t g = c / cig, cl = c - g * cig;
            double acc = 0.0, am = 0.0;
            for (int r = 0; r < R; ++r) {
                const int64_t hp = h + pad - r;
                if (hp < 0 || hp % stride != 0 || hp / stride >= P) continue;
                for (int s = 0; s < S; ++s) {
                    const int64_t wq = w + pad - s;
                    if (wq < 0 || wq % stride != 0 || wq / stride >= Q) continue;
                    for (int64_t k = g * cog; k < (g + 1) * cog; ++k) {
                        double a = load_as_double(dOp, ((b * P + hp / stride) * Q + wq / stride) * C_out + k, dtype);
                        double v = load_as_double(W, ((k * R + r) * S + s) * cig + cl, dtype);
                        acc += a * v;
                        am += (a < 0 ? -a : a) * (v < 0 ? -v : v);
                    }
                }
            }
            dD[t * C_in + c] = acc;
            if (absum) absum[t * C_in + c] = am;
        }
    }
    return 0;
}

/* ---------------------------------------- forward and weight-gradient products */

/*
 * One output pixel of the forward convolution (Sec. II-A, Fig. 1 right, with the
 * filter footprint written out instead of im2col):
 *   O[b,p,q,k] = sum_{r,s,c} D[b, p*stride + r - pad, q*stride + s - pad, c] * W[k,r,s,c]
 * Taps that fall outside the image contribute nothing (zero padding).  Same
 * reading as for the backward product: correlation, dilation 1, one group.
 */
static void fwd_pixel(const void* D, const void* W, int64_t b, int64_t p, int64_t q, int64_t H, int64_t Wd,
                      int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dtype,
                      double* out, double* mag) {
    for (int64_t k = 0; k < C_out; ++k) {
        double acc = 0.0, am = 0.0;
        for (int r = 0; r < R; ++r) {
            int64_t h = p * stride + r - pad;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < S; ++s) {
                int64_t w = q * stride + s - pad;
                if (w < 0 || w >= Wd) continue;
                for (int64_t c = 0; c < C_in; ++c) {
                    double a = load_as_double(D, ((b * H + h) * Wd + w) * C_in + c, dtype);
                    double v = load_as_double(W, ((k * R + r) * S + s) * C_in + c, dtype);
                    acc += a * v;
                    am += (a < 0 ? -a : a) * (v < 0 ? -v : v);
                }
            }
        }
        out[k] = acc;
        if (mag) mag[k] = am;
    }
}

/*
 * Forward pass of a convolution layer: D [B,H,Wd,C_in], W [C_out,R,S,C_in] ->
 * O and absum [B,P,Q,C_out] in fp64.  With pixels != NULL only the output
 * pixels pixels[t] = (b*P + p)*Q + q are computed, as [count, C_out].
 */
int sdgp_ref_conv_fwd(const void* D, const void* W, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                      int64_t C_out, int R, int S, int stride, int pad, int dtype, const int64_t* pixels,
                      int64_t count, double* O, double* absum) {
    if (B < 0 || H < 0 || Wd < 0 || C_in < 0 || C_out < 0 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return -1;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return -1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    const int64_t total = pixels ? count : B * P * Q;
    if (pixels)
        for (int64_t t = 0; t < count; ++t)
            if (pixels[t] < 0 || pixels[t] >= B * P * Q) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < total; ++t) {
        int64_t pix = pixels ? pixels[t] : t;
        int64_t q = pix % Q, p = (pix / Q) % P, b = pix / (Q * P);
        fwd_pixel(D, W, b, p, q, H, Wd, C_in, C_out, R, S, stride, pad, dtype, O + t * C_out,
                  absum ? absum + t * C_out : NULL);
    }
    return 0;
}

/*
 * Weight gradient of the same layer (Sec. II-A, Fig. 1 right: the second product of
 * the backward pass).  Differentiating the forward sum with respect to W gives
 *   dW[k,r,s,c] = sum_{b,p,q} dO[b,p,q,k] * D[b, p*stride + r - pad, q*stride + s - pad, c]
 * over the output pixels whose tap (r,s) lies inside the image.  dO is the
 * UNPRUNED output gradient: Sec. III-A keeps dO for this product and prunes a
 * copy for the data gradient.  dW and absum are [C_out,R,S,C_in] in fp64; the sum
 * runs over b, p, q ascending.  With entries != NULL only the filter elements
 * entries[t] = ((k*R + r)*S + s)*C_in + c are computed, as [count].
 */
int sdgp_ref_conv_bwd_weight(const void* D, const void* dO, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                             int64_t C_out, int R, int S, int stride, int pad, int dtype,
                             const int64_t* entries, int64_t count, double* dW, double* absum) {
    if (B < 0 || H < 0 || Wd < 0 || C_in < 0 || C_out < 0 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return -1;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return -1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    const int64_t nW = C_out * R * S * C_in;
    const int64_t total = entries ? count : nW;
    if (entries)
        for (int64_t t = 0; t < count; ++t)
            if (entries[t] < 0 || entries[t] >= nW) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < total; ++t) {
        int64_t e = entries ? entries[t] : t;
        int64_t c = e % C_in, s = (e / C_in) % S, r = (e / (C_in * S)) % R, k = e / (C_in * S * R);
        double acc = 0.0, am = 0.0;
        for (int64_t b = 0; b < B; ++b)
            for (int64_t p = 0; p < P; ++p) {
                int64_t h = p * stride + r - pad;
                if (h < 0 || h >= H) continue;
                for (int64_t q = 0; q < Q; ++q) {
                    int64_t w = q * stride + s - pad;
                    if (w < 0 || w >= Wd) continue;
                    double g = load_as_double(dO, ((b * P + p) * Q + q) * C_out + k, dtype);
                    double a = load_as_double(D, ((b * H + h) * Wd + w) * C_in + c, dtype);
                    acc += g * a;
                    am += (g < 0 ? -g : g) * (a < 0 ? -a : a);
                }
            }
        dW[t] = acc;
        if (absum) absum[t] = am;
    }
    return 0;
}

/* Number of OpenMP threads the loops above will use (reported by the benchmark). */
#ifdef _OPENMP
#include <omp.h>
int sdgp_ref_threads(void) { return omp_get_max_threads(); }
#else
int sdgp_ref_threads(void) { return 1; }
#endif
