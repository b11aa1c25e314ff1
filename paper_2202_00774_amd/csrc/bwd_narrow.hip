// Backward-data for layers with very few input channels (C_in <= 4: the first convolution of a network); the layer
// is bound by reading dL/dO once.  A workgroup owns a TH x TW tile of input pixels of one image and brings every
// gradient pixel its taps can reach into LDS once, pruning each m-group with the register ranker on the way
// (Sec. III-B; stored dense with zeros).  Four kernels (Fig. 3 left; bf16 storage, fp32 accumulation):
//   * bwd_first_stream (further down), for 3x3 stride-1 padding-1 filters with 64 output channels on even images: the
//     16-column product below, one wavefront streaming a strip of the image through a ring of gradient rows.
//   * bwd_first2 (further down), for 7x7 stride-2 padding-3 filters on even images: a 2 x 2 block of input pixels and
//     their channels are the 16 columns of one small product over a 4 x 4 window of gradient pixels.
//   * bwd_narrow_mm, when the tile's (row tile, column tile) pairs and LDS fit (up to 7x7 filters on RGB): with so few columns per tap the product is turned around.  The matrix
//     cores compute T[gradient pixel][tap, c] = sum_k prune(dL/dO)[pixel][k] W[k][tap][c] -- a plain GEMM with
//     taps x C_in columns (27 for a 3x3 filter on RGB, padded to 32) -- into LDS, and every thread then sums, for
//     its input pixel, the one entry per tap that belongs to it.
//   * bwd_narrow, otherwise: every thread accumulates its own pixel over taps and channels on the vector ALU.
#include "lds_copy.h"

namespace sdgp {

namespace {

constexpr int kNarrowKC = 64;  // output channels per pass through LDS
typedef uint32_t u32x4n __attribute__((ext_vector_type(4)));
typedef float f32x4n __attribute__((ext_vector_type(4)));
#define SDGP_LDSN __attribute__((address_space(3)))

struct NarrowParams {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    int B, H, Wd, P, Q, C_in, C_out, R, S, stride, pad;
    int TH, TW, tiles_h, tiles_w;
    int HP, HQ;  // gradient pixels per tile (rows, columns), upper bound
    int nt;             // 32-column tiles of (tap, c) pairs (matrix-core variant)
    const unsigned char* wimg;  // matrix-core variant: the transposed filter slices as they sit in LDS, one image of
    int wimg_units;             // wimg_units KB per 64 output channels (built once per call in the workspace), or null
    uint32_t hq_magic;  // floor(2^32 / HQ) + 1: x / HQ == umulhi(x, hq_magic) for the pixel counts of a tile
    uint32_t nt_magic;  // floor(2^16 / nt) + 1: x / nt == (x * nt_magic) >> 16 for pair numbers (x < 4096, nt <= 5)
    int n;
    uint32_t mix;
};

constexpr int kAPitchN = kNarrowKC * 2 + 16;  // bytes per gradient pixel in LDS (padded against bank conflicts)

template <int M, int RK, bool PRUNE, bool NLE2>
__global__ void __launch_bounds__(256) bwd_narrow(const NarrowParams p) {
    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDSN unsigned char* smem = (SDGP_LDSN unsigned char*)smem_generic;
    const int tid = threadIdx.x;
    const int tile = blockIdx.x;
    const int tw_i = tile % p.tiles_w, th_i = (tile / p.tiles_w) % p.tiles_h, b = tile / (p.tiles_w * p.tiles_h);
    const int h0 = th_i * p.TH, w0 = tw_i * p.TW;
    // gradient rows/columns the tile's taps can reach: p = (h + pad - r) / stride
    const int lo_h = h0 + p.pad - (p.R - 1), lo_w = w0 + p.pad - (p.S - 1);
    const int pmin = lo_h <= 0 ? 0 : (lo_h + p.stride - 1) / p.stride;
    const int qmin = lo_w <= 0 ? 0 : (lo_w + p.stride - 1) / p.stride;
    const int npix = p.HP * p.HQ;

    SDGP_LDSN unsigned char* lds_a = smem;                                        // [npix][kAPitchN]
    SDGP_LDSN f32x4n* lds_w = (SDGP_LDSN f32x4n*)(smem + ((npix * kAPitchN + 15) & ~15));  // [KC][R*S] x 4 floats

    const int th = tid / p.TW, tw = tid % p.TW;
    const int h = h0 + th, w = w0 + tw;
    const bool live = tid < p.TH * p.TW && h < p.H && w < p.Wd;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int taps = p.R * p.S;

    for (int kc0 = 0; kc0 < p.C_out; kc0 += kNarrowKC) {
        __syncthreads();
        // ---- gradient halo, pruned, into LDS (16 channels per item)
        for (int it = tid; it < npix * (kNarrowKC / 16); it += 256) {
            const int hp = it >> 2, part = it & 3;
            const int pp = pmin + hp / p.HQ, qq = qmin + hp % p.HQ;
            const int k = kc0 + part * 16;
            u32x4n v[2] = {u32x4n{0u, 0u, 0u, 0u}, u32x4n{0u, 0u, 0u, 0u}};
            const bool ok = pp < p.P && qq < p.Q;
            const size_t gp = ok ? ((size_t)(b * p.P + pp) * p.Q + qq) : 0;
            if (ok) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    if (k + i * 8 < p.C_out)
                        v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4n*>(p.dO + gp * p.C_out + k + i * 8));
            }
            if constexpr (PRUNE) {
                uint32_t raw[16], out[16];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        raw[i * 8 + 2 * x] = v[i][x] & 0xFFFFu;
                        raw[i * 8 + 2 * x + 1] = v[i][x] >> 16;
                    }
                const uint64_t e0 = (uint64_t)gp * (uint64_t)p.C_out + (uint64_t)k;
#pragma unroll
                for (int g = 0; g < 16 / M; ++g) {
                    uint32_t r[M], o[M];
                    bool kk[M];
#pragma unroll
                    for (int j = 0; j < M; ++j) r[j] = raw[g * M + j];
                    const uint64_t eg = e0 + (uint64_t)(g * M);
                    prune_group<kBF16, M, RK, NLE2>(r, p.n, hash_row(p.mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
                    for (int j = 0; j < M; ++j) out[g * M + j] = o[j];
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int x = 0; x < 4; ++x) v[i][x] = out[i * 8 + 2 * x] | (out[i * 8 + 2 * x + 1] << 16);
            }
            *(SDGP_LDSN u32x4n*)(lds_a + hp * kAPitchN + part * 32) = v[0];
            *(SDGP_LDSN u32x4n*)(lds_a + hp * kAPitchN + part * 32 + 16) = v[1];
        }
        // ---- filter slice [kc0, kc0+64) x taps x C_in -> fp32, four floats per (k, tap)
        for (int it = tid; it < kNarrowKC * taps; it += 256) {
            const int kk = it / taps, t = it % taps;
            f32x4n wv = {0.f, 0.f, 0.f, 0.f};
            if (kc0 + kk < p.C_out)
                for (int c = 0; c < p.C_in; ++c)
                    wv[c] = bf16_to_float(p.W[((size_t)(kc0 + kk) * taps + t) * p.C_in + c]);
            lds_w[it] = wv;
        }
        __syncthreads();

        if (live) {
            for (int r = 0; r < p.R; ++r) {
                const int hr = h + p.pad - r;
                if (hr < 0 || hr % p.stride != 0) continue;
                const int pp = hr / p.stride;
                if (pp >= p.P) continue;
                for (int s = 0; s < p.S; ++s) {
                    const int ws = w + p.pad - s;
                    if (ws < 0 || ws % p.stride != 0) continue;
                    const int qq = ws / p.stride;
                    if (qq >= p.Q) continue;
                    const int hp = (pp - pmin) * p.HQ + (qq - qmin);
                    const int t = r * p.S + s;
#pragma unroll
                    for (int c8 = 0; c8 < kNarrowKC / 8; ++c8) {
                        const u32x4n a = *(SDGP_LDSN u32x4n*)(lds_a + hp * kAPitchN + c8 * 16);
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            const float lo = __uint_as_float(a[x] << 16), hi = __uint_as_float(a[x] & 0xFFFF0000u);
                            const f32x4n w0v = lds_w[(c8 * 8 + 2 * x) * taps + t];
                            const f32x4n w1v = lds_w[(c8 * 8 + 2 * x + 1) * taps + t];
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[c] = fmaf(lo, w0v[c], fmaf(hi, w1v[c], acc[c]));
                        }
                    }
                }
            }
        }
    }
    if (live) {
        uint16_t* dst = p.dD + ((size_t)(b * p.H + h) * p.Wd + w) * p.C_in;
        for (int c = 0; c < p.C_in; ++c) dst[c] = (uint16_t)float_to_bf16(acc[c]);
    }
}

typedef __bf16 bf16x8n __attribute__((ext_vector_type(8)));
typedef float f32x16n __attribute__((ext_vector_type(16)));

constexpr int kMmRowB = 128;    // bytes per gradient pixel in LDS: 64 channels
constexpr int kMmMaxNt = 5;     // column tiles: up to 160 (tap, c) columns, a 7x7 filter on three channels
constexpr int kMmMaxPairs = 8;  // (32-pixel row tile, 32-column tile) pairs per wavefront: at most 32 per workgroup

// KB of one transposed filter slice in LDS: nt * 32 columns of kAPitchN bytes, rounded up to whole copy units.
constexpr int narrow_image_units(int nt) { return (nt * 32 * kAPitchN + 1023) / 1024; }

// The filter as bwd_narrow_mm wants it in LDS, built once per call: for every slice of 64 output channels the
// columns j = tap * C_in + c with their 64 channels contiguous (kAPitchN bytes per column), zeros in the padding, past
// the last column and past C_out.  One workgroup per slice.
__global__ void __launch_bounds__(256) narrow_w_image(const uint16_t* __restrict__ W, uint16_t* __restrict__ img, int C_out,
                                                      int J, int units) {
    const int kc0 = blockIdx.x * kNarrowKC;
    uint16_t* dst = img + (size_t)blockIdx.x * units * 512;
    constexpr int kPitchE = kAPitchN / 2;
    for (int e = threadIdx.x; e < units * 512; e += 256) {
        const int j = e / kPitchE, kk = e - j * kPitchE;
        uint16_t v = 0;
        if (j < J && kk < kNarrowKC && kc0 + kk < C_out) v = W[(size_t)(kc0 + kk) * J + j];
        dst[e] = v;
    }
}

// One input pixel's sum over the taps that reach it, from the table T of per-pixel, per-(tap, c) products in LDS.
// Tap r reaches row h when h + pad - r is a multiple of the stride: r = r0 + i * stride with the gradient row falling
// by one per step, at most NR steps (NS along the width).  Every read is issued before the first addition; a tap
// outside the filter or the gradient reads T[0..3] and adds nothing.  Same order of additions as the plain loops.
template <int NR, int NS>
__device__ __forceinline__ void narrow_gather(const NarrowParams& p, const SDGP_LDSN float* lds_t, int TP, int pmin, int qmin,
                                              int h, int w, float (&sum)[4]) {
    // (h + pad) = pp0 * stride + r0; strides one and two without the integer division
    const int hp = h + p.pad, wp = w + p.pad;
    int r0, s0, pp0, qq0;
    if (p.stride == 1) {
        r0 = 0, s0 = 0, pp0 = hp, qq0 = wp;
    } else if (p.stride == 2) {
        r0 = hp & 1, s0 = wp & 1, pp0 = hp >> 1, qq0 = wp >> 1;
    } else {
        r0 = hp % p.stride, s0 = wp % p.stride, pp0 = hp / p.stride, qq0 = wp / p.stride;
    }
    int rowoff[NR], coloff[NS];
    bool rv[NR], cv[NS];
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        const int r = r0 + i * p.stride, pp = pp0 - i;
        rv[i] = r < p.R && pp >= 0 && pp < p.P;
        rowoff[i] = (pp - pmin) * p.HQ * TP + r * p.S * p.C_in;
    }
#pragma unroll
    for (int j = 0; j < NS; ++j) {
        const int sx = s0 + j * p.stride, qq = qq0 - j;
        cv[j] = sx < p.S && qq >= 0 && qq < p.Q;
        coloff[j] = (qq - qmin) * TP + sx * p.C_in;
    }
    float v[NR][NS][4];
#pragma unroll
    for (int i = 0; i < NR; ++i)
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const int off = (rv[i] && cv[j]) ? rowoff[i] + coloff[j] : 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[i][j][c] = (c < p.C_in) ? lds_t[off + c] : 0.0f;
        }
#pragma unroll
    for (int i = 0; i < NR; ++i)
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const bool ok = rv[i] && cv[j];
#pragma unroll
            for (int c = 0; c < 4; ++c) sum[c] += ok ? v[i][j][c] : 0.0f;
        }
}

// One 16-channel item of the gradient tile in LDS, in place: positions that are not gradient (outside the image, past
// C_out) are cleared, the rest pruned and stored dense with zeros.
template <int M, int RK, bool PRUNE, bool NLE2>
__device__ __forceinline__ void narrow_item_in_place(const NarrowParams& p, int b, int pmin, int qmin, int kc0, int it,
                                                     SDGP_LDSN unsigned char* lds_a) {
    const int hp = it >> 2, part = it & 3;
    const int hrow = (int)__umulhi((uint32_t)hp, p.hq_magic);
    const int pp = pmin + hrow, qq = qmin + (hp - hrow * p.HQ);
    const int k = kc0 + part * 16;
    const int sw = (hp >> 1) & 7;
    SDGP_LDSN u32x4n* g0 = (SDGP_LDSN u32x4n*)(lds_a + hp * kMmRowB + (((2 * part) ^ sw) << 4));
    SDGP_LDSN u32x4n* g1 = (SDGP_LDSN u32x4n*)(lds_a + hp * kMmRowB + (((2 * part + 1) ^ sw) << 4));
    const u32x4n zero = {0u, 0u, 0u, 0u};
    if (!(pp < p.P && qq < p.Q) || k >= p.C_out) {
        *g0 = zero;
        *g1 = zero;
    } else if (PRUNE || k + 8 >= p.C_out) {
        u32x4n v[2] = {*g0, k + 8 < p.C_out ? *g1 : zero};
        if constexpr (PRUNE) {
            const size_t gp = (size_t)(b * p.P + pp) * p.Q + qq;
            prune16_dense<M, RK, NLE2>(v, p.n, p.mix, (uint64_t)gp * (uint64_t)p.C_out + (uint64_t)k);
        }
        *g0 = v[0];
        *g1 = v[1];
    }
}

// The input pixel (h, w) of image b: sums, from the table T in LDS, the entry of each tap that reaches it -- tap r
// reaches row h when h + pad - r is a multiple of the stride, so r starts at (h + pad) mod stride and steps by the
// stride while the gradient row falls -- and stores the pixel.
__device__ __forceinline__ void narrow_sum_and_store(const NarrowParams& p, const SDGP_LDSN float* lds_t, int TP, int pmin,
                                                     int qmin, int b, int h, int w) {
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
    const int nr = (p.R + p.stride - 1) / p.stride, ns = (p.S + p.stride - 1) / p.stride;  // taps per dimension, at most
    if (nr <= 2 && ns <= 2) {
        narrow_gather<2, 2>(p, lds_t, TP, pmin, qmin, h, w, sum);
    } else if (nr <= 3 && ns <= 3) {
        narrow_gather<3, 3>(p, lds_t, TP, pmin, qmin, h, w, sum);
    } else if (nr <= 4 && ns <= 4) {
        narrow_gather<4, 4>(p, lds_t, TP, pmin, qmin, h, w, sum);
    } else {
        const int r0 = (h + p.pad) % p.stride, s0 = (w + p.pad) % p.stride;
        const int pp0 = (h + p.pad - r0) / p.stride, qq0 = (w + p.pad - s0) / p.stride;
        for (int r = r0, pp = pp0; r < p.R && pp >= 0; r += p.stride, --pp) {
            if (pp >= p.P) continue;
            const SDGP_LDSN float* trow = lds_t + ((pp - pmin) * p.HQ + (qq0 - qmin)) * TP + (r * p.S + s0) * p.C_in;
            for (int s = s0, qq = qq0; s < p.S && qq >= 0; s += p.stride, --qq) {
                if (qq < p.Q)
                    for (int c = 0; c < p.C_in; ++c) sum[c] += trow[c];
                trow += p.stride * p.C_in - TP;  // next tap of this phase, previous gradient pixel
            }
        }
    }
    uint16_t* dst = p.dD + ((size_t)(b * p.H + h) * p.Wd + w) * p.C_in;
    for (int c = 0; c < p.C_in; ++c) dst[c] = (uint16_t)float_to_bf16(sum[c]);
}

// Matrix-core variant; p.nt = 32-column tiles of (tap, c) pairs; kMmPairs = pairs per wavefront (accumulator registers).
template <int M, int RK, bool PRUNE, bool NLE2, int kMmPairs>
__global__ void __launch_bounds__(256, 2) bwd_narrow_mm(const NarrowParams p) {
    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDSN unsigned char* smem = (SDGP_LDSN unsigned char*)smem_generic;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = blockIdx.x;
    const int tw_i = tile % p.tiles_w, th_i = (tile / p.tiles_w) % p.tiles_h, b = tile / (p.tiles_w * p.tiles_h);
    const int h0 = th_i * p.TH, w0 = tw_i * p.TW;
    const int lo_h = h0 + p.pad - (p.R - 1), lo_w = w0 + p.pad - (p.S - 1);
    const int pmin = lo_h <= 0 ? 0 : (lo_h + p.stride - 1) / p.stride;
    const int qmin = lo_w <= 0 ? 0 : (lo_w + p.stride - 1) / p.stride;
    const int npix = p.HP * p.HQ;
    const int nrt = (npix + 31) >> 5;           // row tiles; rows past npix hold whatever LDS held: nobody reads their results
    const int nt = p.nt;
    const int npairs = nrt * nt;
    const int J = p.R * p.S * p.C_in;           // live columns
    const int TP = J | 1;                       // floats per row of T (odd: the gather walks rows)

    // gradient: 128 bytes per pixel (64 channels); 16-byte group g of pixel hp sits at position g ^ ((hp >> 1) & 7),
    // which spreads the fragment reads of 16 consecutive pixels over all banks
    SDGP_LDSN unsigned char* lds_a = smem;                          // [nrt * 32][128]
    SDGP_LDSN unsigned char* lds_wt = smem + nrt * 32 * kMmRowB;    // [nt * 32][kAPitchN]    filter slice, transposed
    SDGP_LDSN float* lds_t = (SDGP_LDSN float*)smem;                // [nrt * 32][TP]         after the last chunk
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    const int nunits = (npix + 7) >> 3;         // copy units: 8 pixels x 128 bytes

    // this wavefront's pairs: wave, wave + 4, ...
    int pair_a[kMmPairs], pair_b[kMmPairs];     // LDS offsets of the pair's row tile and column tile
    int pair_rt[kMmPairs], pair_u[kMmPairs];
#pragma unroll
    for (int i = 0; i < kMmPairs; ++i) {
        const int pr = min(wave + 4 * i, npairs - 1);
        pair_rt[i] = (int)(((uint32_t)pr * p.nt_magic) >> 16), pair_u[i] = pr - pair_rt[i] * nt;
        pair_a[i] = pair_rt[i] * 32 * kMmRowB, pair_b[i] = pair_u[i] * 32 * kAPitchN;
    }
    f32x16n acc[kMmPairs];
#pragma unroll
    for (int i = 0; i < kMmPairs; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;

    for (int kc0 = 0; kc0 < p.C_out; kc0 += kNarrowKC) {
        __syncthreads();
        // ---- gradient halo straight into LDS, every request of the tile in flight at once.  Pixels outside the
        // gradient, the tail of the last unit and channels past C_out copy some valid bytes; the pass below clears them.
        for (int u = wave; u < nunits; u += 4) {
            const int hp = u * 8 + (lane >> 3);
            const int hpc = min(hp, npix - 1);
            const int hrow = (int)__umulhi((uint32_t)hpc, p.hq_magic);
            const int pp = min(pmin + hrow, p.P - 1), qq = min(qmin + (hpc - hrow * p.HQ), p.Q - 1);
            int k = kc0 + (((lane & 7) ^ ((hp >> 1) & 7)) << 3);
            if (k >= p.C_out) k = kc0;
            lds_copy16(p.dO + ((size_t)(b * p.P + pp) * p.Q + qq) * p.C_out + k, smem_base + (uint32_t)u * 1024u);
        }
        // ---- filter slice [kc0, kc0 + 64) x (tap, c), transposed: column j = tap * C_in + c, channels contiguous;
        // copied as it is when the call built the image, else gathered element by element
        if (p.wimg) {
            const unsigned char* src = p.wimg + (size_t)(kc0 / kNarrowKC) * p.wimg_units * 1024;
            for (int u = wave; u < p.wimg_units; u += 4)
                lds_copy16(src + (size_t)u * 1024 + lane * 16, smem_base + (uint32_t)(nrt * 32 * kMmRowB) + (uint32_t)u * 1024u);
        } else {
            constexpr int kPer = kNarrowKC * 32 / 256;  // elements per thread and column tile
            uint16_t wv[kMmMaxNt][kPer];                // every load first, then the LDS writes
#pragma unroll
            for (int u = 0; u < kMmMaxNt; ++u)
#pragma unroll
                for (int i = 0; i < kPer; ++i) {
                    const int it = tid + i * 256;
                    const int kk = it >> 5, j = u * 32 + (it & 31);
                    wv[u][i] = 0;
                    if (u < nt && j < J && kc0 + kk < p.C_out) wv[u][i] = p.W[(size_t)(kc0 + kk) * J + j];
                }
#pragma unroll
            for (int u = 0; u < kMmMaxNt; ++u)
                if (u < nt) {
#pragma unroll
                    for (int i = 0; i < kPer; ++i) {
                        const int it = tid + i * 256;
                        const int kk = it >> 5, j = u * 32 + (it & 31);
                        *(SDGP_LDSN uint16_t*)(lds_wt + j * kAPitchN + kk * 2) = wv[u][i];
                    }
                }
        }
        wait_lds_copies<0>();
        __syncthreads();
        // ---- in place: clear what is not gradient, prune the rest (16 channels per item); nothing to do for a dense
        // tile whose gradient pixels and channels all exist
        const bool all_there = pmin + p.HP <= p.P && qmin + p.HQ <= p.Q && kc0 + kNarrowKC <= p.C_out;
        if (PRUNE || !all_there) {
            for (int it = tid; it < npix * (kNarrowKC / 16); it += 256)
                narrow_item_in_place<M, RK, PRUNE, NLE2>(p, b, pmin, qmin, kc0, it, lds_a);
        }
        __syncthreads();

        // ---- T += gradient x filter slice
        const int bfrag = (lane & 31) * kAPitchN + (lane >> 5) * 16;
        const int arow = (lane & 31) * kMmRowB;                              // row tiles start at multiples of 32 pixels:
        const int aswz = ((lane & 31) >> 1) & 7, ahalf = lane >> 5;          // the swizzle depends on the lane only
#pragma unroll
        for (int ks = 0; ks < kNarrowKC / 16; ++ks) {
#pragma unroll
            for (int i = 0; i < kMmPairs; ++i) {
                if (wave + 4 * i < npairs) {
                    const bf16x8n afr = __builtin_bit_cast(bf16x8n, *(SDGP_LDSN u32x4n*)(lds_a + pair_a[i] + arow + (((2 * ks + ahalf) ^ aswz) << 4)));
                    const bf16x8n bfr = __builtin_bit_cast(bf16x8n, *(SDGP_LDSN u32x4n*)(lds_wt + pair_b[i] + bfrag + ks * 32));
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afr, bfr, acc[i], 0, 0, 0);
                }
            }
        }
    }
    __syncthreads();  // every fragment is read: T takes the place of the gradient
#pragma unroll
    for (int i = 0; i < kMmPairs; ++i) {
        if (wave + 4 * i < npairs) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = pair_rt[i] * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int col = pair_u[i] * 32 + (lane & 31);
                if (col < J) lds_t[row * TP + col] = acc[i][r];
            }
        }
    }
    __syncthreads();

    // ---- every input pixel sums the entry of each tap that reaches it: tap r reaches row h when h + pad - r is a
    // multiple of the stride, so r starts at (h + pad) mod stride and steps by the stride while the gradient row falls
    const int th = tid / p.TW, tw = tid % p.TW;
    const int h = h0 + th, w = w0 + tw;
    if (tid < p.TH * p.TW && h < p.H && w < p.Wd) narrow_sum_and_store(p, lds_t, TP, pmin, qmin, b, h, w);
}

// ---------------------------------------------------------------------------------------------------------------
// 7x7, stride 2, padding 3 on C_in <= 4 (the first layer of an ImageNet ResNet), even image sizes.
//
// An input pixel (2i + a, 2j + b) is reached by the taps r = a + 3 - 2 dp, s = b + 3 - 2 dq of the gradient pixels
// (i + dp, j + dq), dp, dq in [-1, 2].  So the four pixels of a 2 x 2 block and their channels (padded to four) are the
// 16 columns n = (a, b, c) of ONE small product over a 4 x 4 window of gradient pixels,
//   out[(i, j)][n] = sum_{dp, dq} sum_k dO[i + dp, j + dq][k] * V[(dp, dq)][k][n],
// with V the filter re-indexed (zeros where r or s falls outside the filter): rows = gradient-grid positions,
// reduction = 16 window positions x C_out, on v_mfma_f32_16x16x32_bf16 with the result left in registers -- no table
// of per-tap products in LDS, no per-pixel gather.  A lane ends up with the channels of one input pixel.
//   * workgroup = 4 wavefronts, tile = 16 x 32 gradient-grid positions (32 x 64 input pixels: of the tiles of 512
//     positions the one with the smallest halo that keeps two 16-column groups per wavefront); wavefront rq owns grid
//     rows 4 rq .. 4 rq + 3: 4 x 2 accumulators of four registers;
//   * the reduction runs in chunks of 32 channels: the 19 x 35 gradient pixels the tile's windows reach (64 bytes each,
//     80-byte pitch: sixteen consecutive pixels read conflict-free, and every fragment address is a per-lane base plus
//     a constant) and V's chunk (16 window positions x 16 columns, built once per call in the workspace) arrive by
//     direct-to-LDS copies; slots of pixels outside the gradient are cleared once and skipped by the copies; pruning, when asked
//     for, is done in place;
//   * a gradient fragment (16 pixels x 32 channels) is read once per (tile row, dq) and feeds up to four matrix
//     instructions (the output rows whose window holds that gradient row); V's 16 fragments sit in registers.
constexpr int kFWin = 4;                                  // window positions per dimension
constexpr int kFKC = 32;                                  // channels per chunk
constexpr int kFRows = 16, kFCols = 32;                   // tile, in gradient-grid positions
constexpr int kFHaloRows = kFRows + kFWin - 1, kFHaloCols = kFCols + kFWin - 1;
constexpr int kFPix = kFHaloRows * kFHaloCols;            // 665 gradient pixels
constexpr uint32_t kFColMagic = 65536u / kFHaloCols + 1u; // x / kFHaloCols == (x * magic) >> 16 for x < 700
constexpr int kFPitch = 80;                               // bytes per pixel in LDS: 64 of data, 16 of padding
constexpr int kFAUnits = (kFPix * kFPitch + 1023) / 1024; // 1 KB copy units
constexpr int kFABytes = kFAUnits * 1024;
constexpr int kFWRows = kFWin * kFWin * 16;               // rows of V's chunk: (window position, column)
constexpr int kFWUnits = kFWRows * kFPitch / 1024;        // 20
constexpr int kFThreads = 256;
static_assert(kFWRows * kFPitch % 1024 == 0, "V's chunk is whole copy units");

struct FirstParams {
    const uint16_t* dO;
    const unsigned char* vimg;   // [C_out / 32][kFWRows][kFPitch bytes]
    uint16_t* dD;
    int B, P, Q, C_in, C_out;
    int tiles_i, tiles_j;
    int n;
    uint32_t mix;
};

// V's image for one chunk of 32 output channels: row (window position t = (dp+1)*4 + (dq+1), column n = a*8 + b*4 + c),
// 32 channels contiguous, kFPitch bytes per row.  One workgroup per (chunk, window position).
__global__ void __launch_bounds__(256) first_v_image(const uint16_t* __restrict__ W, uint16_t* __restrict__ img, int C_in) {
    const int kc = blockIdx.x >> 4, t = blockIdx.x & 15;
    uint16_t* dst = img + ((size_t)kc * kFWRows + t * 16) * (kFPitch / 2);
    const int dp = (t >> 2) - 1, dq = (t & 3) - 1;
    for (int e = threadIdx.x; e < 16 * (kFPitch / 2); e += 256) {
        const int nn = e / (kFPitch / 2), kk = e % (kFPitch / 2);
        const int a = nn >> 3, b = (nn >> 2) & 1, c = nn & 3;
        const int r = a + 3 - 2 * dp, s2 = b + 3 - 2 * dq;
        uint16_t v = 0;
        if (kk < kFKC && c < C_in && r >= 0 && r < 7 && s2 >= 0 && s2 < 7)
            v = W[(((size_t)(kc * kFKC + kk) * 7 + r) * 7 + s2) * C_in + c];
        dst[e] = v;
    }
}

typedef float f32x4f __attribute__((ext_vector_type(4)));

template <int M, int RK, bool PRUNE, bool NLE2>
__global__ void __launch_bounds__(kFThreads, 2) bwd_first2(const FirstParams p) {
    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDSN unsigned char* smem = (SDGP_LDSN unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rq = wave, gp = 0;
    const int tile = blockIdx.x;
    const int tj = tile % p.tiles_j, ti = (tile / p.tiles_j) % p.tiles_i, b = tile / (p.tiles_j * p.tiles_i);
    const int i0 = ti * kFRows, j0 = tj * kFCols;
    const int px = lane & 15, oct = lane >> 4;

    f32x4f acc[4][2];
#pragma unroll
    for (int ri = 0; ri < 4; ++ri)
#pragma unroll
        for (int g = 0; g < 2; ++g) acc[ri][g] = f32x4f{0.f, 0.f, 0.f, 0.f};

    // this lane's bases: V fragments (row = window position * 16 + column px), gradient fragments (tile row 4 rq,
    // column 32 gp + px, window column 0)
    SDGP_LDSN unsigned char* const vbase = smem + kFABytes + px * kFPitch + oct * 16;
    SDGP_LDSN unsigned char* const abase = smem + ((4 * rq) * kFHaloCols + 32 * gp + px) * kFPitch + oct * 16;

    // Where this lane's 16-byte slots of the gradient tile come from: a byte offset inside image b (the same for every
    // chunk, which only moves the base by 64 bytes), or "nothing" -- padding slots, slots past the tile, pixels outside
    // the gradient.  The latter are cleared once; the copies skip them.
    constexpr int kUnitsPerWave = (kFAUnits + 3) / 4;
    constexpr uint32_t kNothing = 0xFFFFFFFFu;
    uint32_t voff[kUnitsPerWave];
#pragma unroll
    for (int x = 0; x < kUnitsPerWave; ++x) {
        const int u = wave + 4 * x;
        const int slot = u * 64 + lane;                                  // 16-byte slot of the tile
        const int pix = (int)(((uint32_t)slot * 13108u) >> 16);          // slot / 5
        const int part = slot - 5 * pix;                                 // 0..3 data, 4 padding
        const int hr = (int)(((uint32_t)pix * kFColMagic) >> 16);        // pix / kFHaloCols
        const int gi = i0 - 1 + hr, gj = j0 - 1 + (pix - hr * kFHaloCols);
        const bool ok = u < kFAUnits && part < 4 && pix < kFPix && gi >= 0 && gi < p.P && gj >= 0 && gj < p.Q;
        voff[x] = ok ? (uint32_t)((gi * p.Q + gj) * p.C_out + part * 8) * 2u : kNothing;
        if (!ok && u < kFAUnits) *(SDGP_LDSN u32x4n*)(smem + slot * 16) = u32x4n{0u, 0u, 0u, 0u};
    }
    const unsigned char* const image = reinterpret_cast<const unsigned char*>(p.dO + (size_t)b * p.P * p.Q * p.C_out);

    const int nchunks = p.C_out / kFKC;
    for (int kc = 0; kc < nchunks; ++kc) {
        if (kc > 0) __syncthreads();   // the previous chunk's fragments are read
#pragma unroll
        for (int x = 0; x < kUnitsPerWave; ++x) {
            const int u = wave + 4 * x;
            if (voff[x] != kNothing) lds_copy16(image + (size_t)kc * (kFKC * 2), voff[x], smem_base + (uint32_t)u * 1024u);
        }
        for (int u = wave; u < kFWUnits; u += 4)
            lds_copy16(p.vimg + ((size_t)kc * kFWUnits + u) * 1024 + lane * 16, smem_base + (uint32_t)(kFABytes + u * 1024));
        wait_lds_copies<0>();
        __syncthreads();
        if constexpr (PRUNE) {
            for (int it = tid; it < kFPix * 2; it += kFThreads) {
                const int hp = it >> 1, half = it & 1;
                const int hr = (int)(((uint32_t)hp * kFColMagic) >> 16);
                const int gi = i0 - 1 + hr, gj = j0 - 1 + (hp - hr * kFHaloCols);
                if (gi >= 0 && gi < p.P && gj >= 0 && gj < p.Q) {
                    SDGP_LDSN u32x4n* g0 = (SDGP_LDSN u32x4n*)(smem + hp * kFPitch + half * 32);
                    u32x4n v[2] = {g0[0], g0[1]};
                    const size_t gpix = (size_t)(b * p.P + gi) * p.Q + gj;
                    prune16_dense<M, RK, NLE2>(v, p.n, p.mix, (uint64_t)gpix * (uint64_t)p.C_out + (uint64_t)(kc * kFKC + half * 16));
                    g0[0] = v[0];
                    g0[1] = v[1];
                }
            }
            __syncthreads();
        }
        bf16x8n vf[kFWin * kFWin];
#pragma unroll
        for (int t = 0; t < kFWin * kFWin; ++t) vf[t] = __builtin_bit_cast(bf16x8n, *(SDGP_LDSN u32x4n*)(vbase + t * 16 * kFPitch));
#pragma unroll
        for (int rr = 0; rr < 4 + kFWin - 1; ++rr) {       // gradient rows of this wavefront's four output rows
#pragma unroll
            for (int dqi = 0; dqi < kFWin; ++dqi) {
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const bf16x8n gf = __builtin_bit_cast(bf16x8n, *(SDGP_LDSN u32x4n*)(abase + (rr * kFHaloCols + 16 * g + dqi) * kFPitch));
#pragma unroll
                    for (int ri = 0; ri < 4; ++ri) {
                        const int dpi = rr - ri;             // window row of gradient row rr for output row ri
                        if (dpi >= 0 && dpi < kFWin)
                            acc[ri][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dpi * kFWin + dqi], gf, acc[ri][g], 0, 0, 0);
                    }
                }
            }
        }
    }
    // result register c of lane (px, oct = 2 a + b): channel c of input pixel (2 i + a, 2 j + b)
    const int a = oct >> 1, bb = oct & 1;
#pragma unroll
    for (int ri = 0; ri < 4; ++ri)
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const int i = i0 + 4 * rq + ri, j = j0 + 32 * gp + 16 * g + px;
            if (i < p.P && j < p.Q) {
                uint16_t* dst = p.dD + ((size_t)(b * 2 * p.P + 2 * i + a) * (2 * p.Q) + 2 * j + bb) * p.C_in;
                const uint32_t c01 = float2_to_bf16x2(acc[ri][g][0], acc[ri][g][1]), c23 = float2_to_bf16x2(acc[ri][g][2], acc[ri][g][3]);
                dst[0] = (uint16_t)c01;
                if (p.C_in > 1) dst[1] = (uint16_t)(c01 >> 16);
                if (p.C_in > 2) dst[2] = (uint16_t)c23;
                if (p.C_in > 3) dst[3] = (uint16_t)(c23 >> 16);
            }
        }
}

// Whether bwd_first2 takes the problem (everything but the workspace).
bool first2_fits(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n, int m) {
    if (R != 7 || S != 7 || stride != 2 || pad != 3 || C_in < 1 || C_in > 4 || C_out < kFKC || C_out % kFKC != 0) return false;
    if ((H & 1) || (Wd & 1) || H < 2 || Wd < 2) return false;
    if (n != m && !(m == 4 || m == 8 || m == 16)) return false;
    const int64_t P = H / 2, Q = Wd / 2;   // (H + 6 - 7) / 2 + 1 for even H
    const int64_t tiles = B * ((P + kFRows - 1) / kFRows) * ((Q + kFCols - 1) / kFCols);
    return tiles > 0 && tiles < INT32_MAX && B * H * Wd < INT32_MAX && P * Q * C_out < ((int64_t)1 << 30);
}

size_t first2_image_bytes(int64_t C_out) { return (size_t)(C_out / kFKC) * kFWRows * kFPitch; }

template <int M, int RK, bool PRUNE, bool NLE2>
int launch_first2(const FirstParams& p, hipStream_t stream) {
    auto kern = bwd_first2<M, RK, PRUNE, NLE2>;
    constexpr int lds = kFABytes + kFWRows * kFPitch;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.B * p.tiles_i * p.tiles_j)), dim3(kFThreads), lds, stream, p);
    return launch_status();
}

template <int M, bool NLE2>
int launch_first2_rk(const FirstParams& p, int rk, hipStream_t stream) {
    if (rk == kRandom) return launch_first2<M, kRandom, true, NLE2>(p, stream);
    if (rk == kGreedy) return launch_first2<M, kGreedy, true, NLE2>(p, stream);
    return launch_first2<M, kAdjusted, true, NLE2>(p, stream);
}

// ---------------------------------------------------------------------------------------------------------------
// 3x3, stride 1, padding 1 on C_in <= 4 with 64 output channels (the first layer of a CIFAR-style network), even image
// sizes: the stem kernel's 16-column product, streamed.  Input pixel (2i + a, 2j + b) is reached by tap
// (a + 1 - du, b + 1 - dv) of gradient pixel (2i + du, 2j + dv), du, dv in [-1, 2]: a 4 x 4 window on the gradient,
// 16 columns (a, b, c), rows = 16 consecutive blocks j of one block row i.  The layer is bound by reading the
// gradient once, and a tile kernel keeps the memory system idle whenever its workgroups compute in step; so here
// every WAVEFRONT streams on its own: it owns a strip of 16 blocks (32 input columns) and a range of block rows of
// one image, keeps eight gradient rows in a ring in LDS (4352 bytes each: both 32-channel halves, even and odd
// columns apart so that the 16 lanes of a fragment read neighbours, 16-byte parts permuted by bits 2..3 of the
// record number), computes block row i from rows 2i-1 .. 2i+2 while the rows of the next three block rows are in
// flight, and never meets a barrier after the filter is in place.  The copies are counted: every block row issues
// the same ten instructions (rows or columns outside the image copy from a block of zeros), so "all but the youngest
// 20" is exactly "the rows of this block row have landed".
//   * the filter's fragments are built in the kernel: W is copied transposed into LDS ([tap, c][k], 144-byte pitch)
//     and a fragment is one 16-byte read (or zeros where the tap falls outside the filter);
//   * pruning: a block row prunes the two rows that are new to it, in place, before reading fragments: every
//     gradient row is ranked once per wavefront that streams it (rows shared by two row ranges twice).
constexpr int kSRowBytes = 4352;                          // 68 records of 64 bytes: [half][column parity][17]
constexpr int kSRing = 8;                                 // gradient rows per wavefront
constexpr int kSRingBytes = kSRing * kSRowBytes;
constexpr int kSCopiesPerRow = 5;                         // 272 sixteen-byte slots: four full instructions and 16 lanes
constexpr int kSWPitch = 144;                             // bytes per (tap, c) row of the transposed filter
constexpr int kSLds = 4 * kSRingBytes + 36 * kSWPitch;

__device__ __align__(64) const uint32_t kStreamZeros[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

struct StreamParams {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    int B, H, Wd, C_in;
    int strips, splits, steps_per_split;   // column strips per image, row ranges per strip, block rows per range
    int tasks;                             // B * strips * splits
    int n;
    uint32_t mix;
};

template <int M, int RK, bool PRUNE, bool NLE2>
__global__ void __launch_bounds__(256, 1) bwd_first_stream(const StreamParams p) {
    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDSN unsigned char* smem = (SDGP_LDSN unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int px = lane & 15, oct = lane >> 4;
    const int task = blockIdx.x * 4 + wave;
    const bool active = task < p.tasks;                       // (an idle wavefront still helps with the filter)
    const int split = task % p.splits, strip = (task / p.splits) % p.strips, b = task / (p.splits * p.strips);
    const int nblockrows = p.H >> 1;
    const int i_begin = split * p.steps_per_split;
    const int i_end = active ? min(i_begin + p.steps_per_split, nblockrows) : i_begin;
    const int j0 = strip * 16;                                // first block of the strip
    const int q0 = 2 * j0 - 1;                                // gradient column of record column 0
    const uint32_t ring = smem_base + (uint32_t)wave * kSRingBytes;
    SDGP_LDSN unsigned char* const ringp = smem + wave * kSRingBytes;

    // ---- where this lane's slots of a row come from: byte offset inside the gradient row, or "zeros"
    uint32_t src_off[kSCopiesPerRow];
    bool src_ok[kSCopiesPerRow];
#pragma unroll
    for (int k = 0; k < kSCopiesPerRow; ++k) {
        const int slot = k * 64 + lane;                       // 16-byte slot of the row (272 of them)
        const int rec = slot >> 2;
        const int part = (slot & 3) ^ ((rec >> 2) & 3);       // which eight channels of the half sit here
        const int half = rec >= 34 ? 1 : 0, rem = rec - 34 * half;
        const int plane = rem >= 17 ? 1 : 0, idx = rem - 17 * plane;
        const int q = q0 + 2 * idx + plane;
        src_ok[k] = slot < 272 && q >= 0 && q < p.Wd;
        src_off[k] = (uint32_t)(q * 64 + half * 32 + part * 8) * 2u;
    }
    const unsigned char* const image = reinterpret_cast<const unsigned char*>(p.dO) + (size_t)b * p.H * p.Wd * 128u;
    const unsigned char* const zeros = reinterpret_cast<const unsigned char*>(kStreamZeros);
    const size_t row_bytes = (size_t)p.Wd * 128u;
    // the two (or four) gradient rows that are new to block row i: gradient row r goes to ring slot (r + 1) & 7
    auto issue_row = [&](int r) {
        const bool row_ok = r >= 0 && r < p.H;
        const unsigned char* base = image + (size_t)(row_ok ? r : 0) * row_bytes;
        const uint32_t dst = ring + (uint32_t)((r + 1) & 7) * kSRowBytes;
#pragma unroll
        for (int k = 0; k < kSCopiesPerRow; ++k) {
            const unsigned char* src = (row_ok && src_ok[k]) ? base + src_off[k] : zeros;
            if (k < 4 || lane < 16) lds_copy16(src, dst + (uint32_t)k * 1024u);
        }
    };
    auto issue_step = [&](int i, bool first) {
        if (first) issue_row(2 * i - 1), issue_row(2 * i);
        issue_row(2 * i + 1), issue_row(2 * i + 2);
    };
    if (active) {
        issue_step(i_begin, true);
        if (i_begin + 1 < i_end) issue_step(i_begin + 1, false);
        if (i_begin + 2 < i_end) issue_step(i_begin + 2, false);
    }

    // ---- the filter, transposed: row (tap, c), 64 output channels contiguous
    SDGP_LDSN unsigned char* const wt = smem + 4 * kSRingBytes;
    const int wcols = 9 * p.C_in;
    for (int e = tid; e < 64 * wcols; e += 256) {
        const int k = e / wcols, rsc = e - k * wcols;
        *(SDGP_LDSN uint16_t*)(wt + rsc * kSWPitch + k * 2) = p.W[e];
    }
    __syncthreads();
    if (!active) return;
    bf16x8n vf[2][16];
    {
        const int a = px >> 3, bb = (px >> 2) & 1, c = px & 3;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int r = a + 1 - ((t >> 2) - 1), s2 = bb + 1 - ((t & 3) - 1);
            const bool ok = r >= 0 && r < 3 && s2 >= 0 && s2 < 3 && c < p.C_in;
            const int row = ok ? (r * 3 + s2) * p.C_in + c : 0;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                u32x4n v = *(SDGP_LDSN u32x4n*)(wt + row * kSWPitch + half * 64 + oct * 16);
                if (!ok) v = u32x4n{0u, 0u, 0u, 0u};
                vf[half][t] = __builtin_bit_cast(bf16x8n, v);
            }
        }
    }
    // this lane's fragment of (half, window column dv): record (half, parity of dv, px + dv / 2), part oct
    uint32_t frag_off[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int dv = 0; dv < 4; ++dv) {
            const int rec = (half * 2 + (dv & 1)) * 17 + (dv >> 1) + px;
            frag_off[half][dv] = (uint32_t)(rec * 64 + ((oct ^ ((rec >> 2) & 3)) << 4));
        }

    const int a = oct >> 1, bb = oct & 1;
    for (int i = i_begin; i < i_end; ++i) {
        // the rows of block rows i + 1 and i + 2 (ten copies each) may still be in flight.  (The stores of earlier block
        // rows are in the same counter; not counting them only makes the wait stricter.)
        const int ahead = i_end - 1 - i;
        if (ahead >= 2) wait_lds_copies<20>();
        else if (ahead == 1) wait_lds_copies<10>();
        else wait_lds_copies<0>();
        // (the copies, and below the in-place pruning, hand data from lane to lane through LDS inside one wavefront:
        // the hardware keeps a wavefront's LDS operations in order, the fences keep the compiler from reordering them)
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if constexpr (PRUNE) {
            // the rows new to this block row: up to 34 pixels (the strip's 32 and a neighbour each side where the image
            // goes on) x 4 items of 16 channels.  Every lane ranks an item in every round (straight-line code lets the
            // compiler interleave the rounds); lanes past the last item redo it and do not store.
            const int r_first = i == i_begin ? 2 * i - 1 : 2 * i + 1;
            const int col_first = q0 < 0 ? 1 : 0;
            const int ncols = min(34, p.Wd - q0) - col_first;          // record columns that are gradient pixels
            const int nitems = 4 * ncols;
            for (int r = r_first; r <= 2 * i + 2; ++r) {
                if (r < 0 || r >= p.H) continue;
                SDGP_LDSN unsigned char* const rowp = ringp + ((r + 1) & 7) * kSRowBytes;
                const size_t gpix0 = ((size_t)b * p.H + r) * p.Wd + q0;
                for (int it0 = 0; it0 < nitems; it0 += 128) {
                    SDGP_LDSN u32x4n* g0[2];
                    SDGP_LDSN u32x4n* g1[2];
                    u32x4n v[2][2];
                    bool live[2];
#pragma unroll
                    for (int x = 0; x < 2; ++x) {
                        const int it = it0 + x * 64 + lane;
                        live[x] = it < nitems;
                        const int itc = live[x] ? it : nitems - 1;
                        const int col = (itc >> 2) + col_first, half = (itc >> 1) & 1, sixteen = itc & 1;
                        const int rec = (half * 2 + (col & 1)) * 17 + (col >> 1);
                        const int sw = (rec >> 2) & 3;
                        g0[x] = (SDGP_LDSN u32x4n*)(rowp + rec * 64 + (((2 * sixteen) ^ sw) << 4));
                        g1[x] = (SDGP_LDSN u32x4n*)(rowp + rec * 64 + (((2 * sixteen + 1) ^ sw) << 4));
                        v[x][0] = *g0[x], v[x][1] = *g1[x];
                        prune16_dense<M, RK, NLE2>(v[x], p.n, p.mix, (uint64_t)(gpix0 + col) * 64u + (uint64_t)(half * 32 + sixteen * 16));
                    }
#pragma unroll
                    for (int x = 0; x < 2; ++x)
                        if (live[x]) *g0[x] = v[x][0], *g1[x] = v[x][1];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        f32x4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int du = 0; du < 4; ++du) {
            SDGP_LDSN unsigned char* const rowp = ringp + ((2 * i + du) & 7) * kSRowBytes;   // gradient row 2i - 1 + du
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int dv = 0; dv < 4; ++dv) {
                    const bf16x8n gf = __builtin_bit_cast(bf16x8n, *(SDGP_LDSN u32x4n*)(rowp + frag_off[half][dv]));
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[half][du * 4 + dv], gf, acc, 0, 0, 0);
                }
        }
        // result register c of lane (px, oct = 2 a + b): channel c of input pixel (2 i + a, 2 (j0 + px) + b)
        const int h = 2 * i + a, w = 2 * (j0 + px) + bb;
        if (w < p.Wd) {
            uint16_t* dst = p.dD + (((size_t)b * p.H + h) * p.Wd + w) * p.C_in;
            const uint32_t c01 = float2_to_bf16x2(acc[0], acc[1]), c23 = float2_to_bf16x2(acc[2], acc[3]);
            dst[0] = (uint16_t)c01;
            if (p.C_in > 1) dst[1] = (uint16_t)(c01 >> 16);
            if (p.C_in > 2) dst[2] = (uint16_t)c23;
            if (p.C_in > 3) dst[3] = (uint16_t)(c23 >> 16);
        }
        // rows 2i - 1 and 2i are done with: their ring slots take the rows of block row i + 3
        if (i + 3 < i_end) {
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this block row's fragment reads have returned
            issue_step(i + 3, false);
        }
    }
}

bool stream_fits(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n, int m) {
    if (R != 3 || S != 3 || stride != 1 || pad != 1 || C_in < 1 || C_in > 4 || C_out != 64) return false;
    if ((H & 1) || (Wd & 1) || H < 2 || Wd < 2 || B < 1) return false;
    if (n != m && !(m == 4 || m == 8 || m == 16)) return false;
    return B * ((Wd + 31) / 32) * (H / 2) < (1 << 28) && B * H * Wd < INT32_MAX;
}

template <int M, int RK, bool PRUNE, bool NLE2>
int launch_stream(const StreamParams& p, hipStream_t stream) {
    auto kern = bwd_first_stream<M, RK, PRUNE, NLE2>;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kSLds);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)((p.tasks + 3) / 4)), dim3(256), kSLds, stream, p);
    return launch_status();
}

template <int M, bool NLE2>
int launch_stream_rk(const StreamParams& p, int rk, hipStream_t stream) {
    if (rk == kRandom) return launch_stream<M, kRandom, true, NLE2>(p, stream);
    if (rk == kGreedy) return launch_stream<M, kGreedy, true, NLE2>(p, stream);
    return launch_stream<M, kAdjusted, true, NLE2>(p, stream);
}

// ---------------------------------------------------------------------------------------------------------------
// The same streaming scheme for the 7x7 stride-2 padding-3 stem (C_in <= 3, 64 output channels, even image sizes).
// Block (i, j) = input pixels (2i + a, 2j + b); its window is gradient pixels (i + dp, j + dq), dp, dq in [-1, 2], on a
// gradient grid as coarse as the block grid: block row i needs gradient rows i-1 .. i+2 and every step brings ONE
// new row.  A wavefront owns a strip of 16 blocks (19 gradient columns) and a range of block rows, with a ring of
// seven rows of 2560 bytes ([half][20 records of 64 bytes], parts permuted by bits 2..3 of the record number): four in
// use, three in flight.  Eight wavefronts per workgroup, one workgroup per CU (two wavefronts per SIMD); the filter is
// copied transposed into LDS ([tap, c][k], 128 bytes per row) and a fragment is one 16-byte read.
constexpr int kTRowBytes = 2560;
constexpr int kTRing = 7;
constexpr int kTRingBytes = kTRing * kTRowBytes;
constexpr int kTWaves = 8;
constexpr int kTCopiesPerRow = 3;                         // 160 sixteen-byte slots: two full instructions and 32 lanes
constexpr int kTWRowBytes = 128;
constexpr int kTLds = kTWaves * kTRingBytes + 147 * kTWRowBytes;

struct StemStreamParams {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    int B, P, Q, C_in;                     // P x Q gradient pixels = blocks; the image is 2P x 2Q
    int strips, splits, steps_per_split;
    int tasks;
    int n;
    uint32_t mix;
};

template <int M, int RK, bool PRUNE, bool NLE2>
__global__ void __launch_bounds__(kTWaves * 64, 1) bwd_stem_stream(const StemStreamParams p) {
    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDSN unsigned char* smem = (SDGP_LDSN unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int px = lane & 15, oct = lane >> 4;
    const int task = blockIdx.x * kTWaves + wave;
    const bool active = task < p.tasks;
    const int split = task % p.splits, strip = (task / p.splits) % p.strips, b = task / (p.splits * p.strips);
    const int i_begin = split * p.steps_per_split;
    const int i_end = active ? min(i_begin + p.steps_per_split, p.P) : i_begin;
    const int j0 = strip * 16;
    const int q0 = j0 - 1;                                    // gradient column of record column 0
    const uint32_t ring = smem_base + (uint32_t)wave * kTRingBytes;
    SDGP_LDSN unsigned char* const ringp = smem + wave * kTRingBytes;

    uint32_t src_off[kTCopiesPerRow];
    bool src_ok[kTCopiesPerRow];
#pragma unroll
    for (int k = 0; k < kTCopiesPerRow; ++k) {
        const int slot = k * 64 + lane;                       // 16-byte slot of the row (160 of them)
        const int rec = slot >> 2;
        const int part = (slot & 3) ^ ((rec >> 2) & 3);
        const int half = rec >= 20 ? 1 : 0, x = rec - 20 * half;
        const int q = q0 + x;
        src_ok[k] = slot < 160 && x < 19 && q >= 0 && q < p.Q;
        src_off[k] = (uint32_t)(q * 64 + half * 32 + part * 8) * 2u;
    }
    const unsigned char* const image = reinterpret_cast<const unsigned char*>(p.dO) + (size_t)b * p.P * p.Q * 128u;
    const unsigned char* const zeros = reinterpret_cast<const unsigned char*>(kStreamZeros);
    const size_t row_bytes = (size_t)p.Q * 128u;
    // rows are issued in ascending order into consecutive ring slots; row i_begin - 1 sits in slot 0
    int next_row = i_begin - 1, next_slot = 0;
    auto issue_row = [&]() {
        const int r = next_row;
        const bool row_ok = r >= 0 && r < p.P;
        const unsigned char* base = image + (size_t)(row_ok ? r : 0) * row_bytes;
        const uint32_t dst = ring + (uint32_t)next_slot * kTRowBytes;
#pragma unroll
        for (int k = 0; k < kTCopiesPerRow; ++k) {
            const unsigned char* src = (row_ok && src_ok[k]) ? base + src_off[k] : zeros;
            if (k < 2 || lane < 32) lds_copy16(src, dst + (uint32_t)k * 1024u);
        }
        ++next_row;
        next_slot = next_slot == kTRing - 1 ? 0 : next_slot + 1;
    };
    const int last_row = i_end + 1;                           // the last block row reads gradient row i_end - 1 + 2
    if (active)
        for (int k = 0; k < kTRing && next_row <= last_row; ++k) issue_row();

    // ---- the filter, transposed: row (tap, c), 64 output channels contiguous
    SDGP_LDSN unsigned char* const wt = smem + kTWaves * kTRingBytes;
    const int wcols = 49 * p.C_in;
    for (int e = tid; e < 64 * wcols; e += kTWaves * 64) {
        const int k = e / wcols, rsc = e - k * wcols;
        *(SDGP_LDSN uint16_t*)(wt + rsc * kTWRowBytes + k * 2) = p.W[e];
    }
    __syncthreads();
    if (!active) return;
    bf16x8n vf[2][16];
    {
        const int a = px >> 3, bb = (px >> 2) & 1, c = px & 3;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int r = a + 3 - 2 * ((t >> 2) - 1), s2 = bb + 3 - 2 * ((t & 3) - 1);
            const bool ok = r >= 0 && r < 7 && s2 >= 0 && s2 < 7 && c < p.C_in;
            const int row = ok ? (r * 7 + s2) * p.C_in + c : 0;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                u32x4n v = *(SDGP_LDSN u32x4n*)(wt + row * kTWRowBytes + half * 64 + oct * 16);
                if (!ok) v = u32x4n{0u, 0u, 0u, 0u};
                vf[half][t] = __builtin_bit_cast(bf16x8n, v);
            }
        }
    }
    uint32_t frag_off[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int dq = 0; dq < 4; ++dq) {
            const int rec = half * 20 + dq + px;
            frag_off[half][dq] = (uint32_t)(rec * 64 + ((oct ^ ((rec >> 2) & 3)) << 4));
        }
    const int col_first = q0 < 0 ? 1 : 0;
    const int ncols = min(19, p.Q - q0) - col_first;          // record columns that are gradient pixels
    const int nitems = 4 * ncols;

    const int a = oct >> 1, bb = oct & 1;
    int cslot = 0;                                            // ring slot of gradient row i - 1
    for (int i = i_begin; i < i_end; ++i) {
        // rows up to i + 2 must have landed; up to three younger rows (three copies each) may be in flight
        const int younger = min(next_row - 1, last_row) - (i + 2);
        if (younger >= 3) wait_lds_copies<9>();
        else if (younger == 2) wait_lds_copies<6>();
        else if (younger == 1) wait_lds_copies<3>();
        else wait_lds_copies<0>();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if constexpr (PRUNE) {
            // the rows new to this block row (all four for the first one): up to 19 pixels x 4 items of 16 channels
            const int u_first = i == i_begin ? 0 : 3;
            for (int u = u_first; u < 4; ++u) {
                const int r = i - 1 + u;
                if (r < 0 || r >= p.P) continue;
                int sl = cslot + u;
                sl = sl >= kTRing ? sl - kTRing : sl;
                SDGP_LDSN unsigned char* const rowp = ringp + sl * kTRowBytes;
                const size_t gpix0 = ((size_t)b * p.P + r) * p.Q + q0;
                for (int it0 = 0; it0 < nitems; it0 += 64) {
                    const int it = it0 + lane;
                    const bool live = it < nitems;
                    const int itc = live ? it : nitems - 1;
                    const int col = (itc >> 2) + col_first, half = (itc >> 1) & 1, sixteen = itc & 1;
                    const int rec = half * 20 + col;
                    const int sw = (rec >> 2) & 3;
                    SDGP_LDSN u32x4n* g0 = (SDGP_LDSN u32x4n*)(rowp + rec * 64 + (((2 * sixteen) ^ sw) << 4));
                    SDGP_LDSN u32x4n* g1 = (SDGP_LDSN u32x4n*)(rowp + rec * 64 + (((2 * sixteen + 1) ^ sw) << 4));
                    u32x4n v[2] = {*g0, *g1};
                    prune16_dense<M, RK, NLE2>(v, p.n, p.mix, (uint64_t)(gpix0 + col) * 64u + (uint64_t)(half * 32 + sixteen * 16));
                    if (live) *g0 = v[0], *g1 = v[1];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        f32x4f acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int sl = cslot + u;
            sl = sl >= kTRing ? sl - kTRing : sl;
            SDGP_LDSN unsigned char* const rowp = ringp + sl * kTRowBytes;
#pragma unroll
            for (int dq = 0; dq < 4; ++dq) {
                const bf16x8n g0 = __builtin_bit_cast(bf16x8n, *(SDGP_LDSN u32x4n*)(rowp + frag_off[0][dq]));
                const bf16x8n g1 = __builtin_bit_cast(bf16x8n, *(SDGP_LDSN u32x4n*)(rowp + frag_off[1][dq]));
                acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[0][u * 4 + dq], g0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[1][u * 4 + dq], g1, acc1, 0, 0, 0);
            }
        }
        const f32x4f acc = acc0 + acc1;
        const int h = 2 * i + a, w = 2 * (j0 + px) + bb;
        if (j0 + px < p.Q) {
            uint16_t* dst = p.dD + (((size_t)b * 2 * p.P + h) * (2 * p.Q) + w) * p.C_in;
            const uint32_t c01 = float2_to_bf16x2(acc[0], acc[1]), c23 = float2_to_bf16x2(acc[2], acc[3]);
            dst[0] = (uint16_t)c01;
            if (p.C_in > 1) dst[1] = (uint16_t)(c01 >> 16);
            if (p.C_in > 2) dst[2] = (uint16_t)c23;
        }
        // row i - 1 is done with: its ring slot takes the next row
        cslot = cslot == kTRing - 1 ? 0 : cslot + 1;
        if (next_row <= last_row) {
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this block row's fragment reads have returned
            issue_row();
        }
    }
}

bool stem_stream_fits(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n, int m) {
    if (R != 7 || S != 7 || stride != 2 || pad != 3 || C_in < 1 || C_in > 3 || C_out != 64) return false;
    if ((H & 1) || (Wd & 1) || H < 2 || Wd < 2 || B < 1) return false;
    if (n != m && !(m == 4 || m == 8 || m == 16)) return false;
    return B * ((Wd / 2 + 15) / 16) * (H / 2) < (1 << 28) && B * H * Wd < INT32_MAX;
}

template <int M, int RK, bool PRUNE, bool NLE2>
int launch_stem_stream(const StemStreamParams& p, hipStream_t stream) {
    auto kern = bwd_stem_stream<M, RK, PRUNE, NLE2>;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kTLds);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)((p.tasks + kTWaves - 1) / kTWaves)), dim3(kTWaves * 64), kTLds, stream, p);
    return launch_status();
}

// LDS bytes of bwd_narrow_mm for a tile of npix gradient pixels, nt column tiles and J live columns.
int narrow_mm_lds(int npix, int nt, int J) {
    const int rows = ((npix + 31) / 32) * 32;
    const int loop = rows * kMmRowB + narrow_image_units(nt) * 1024;  // the filter slice in whole copy units
    const int t = rows * (J | 1) * 4;
    return loop > t ? loop : t;
}

template <int M, int RK, bool PRUNE, bool NLE2>
int launch_narrow_mm(const NarrowParams& p, int grid, hipStream_t stream) {
    const int lds = narrow_mm_lds(p.HP * p.HQ, p.nt, p.R * p.S * p.C_in);
    const int npairs = ((p.HP * p.HQ + 31) / 32) * p.nt;
#define SDGP_NARROW_MM(PAIRS)                                                                                         \
    {                                                                                                                 \
        auto kern = bwd_narrow_mm<M, RK, PRUNE, NLE2, PAIRS>;                                                         \
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                       \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);   \
        if (attr != hipSuccess) return SDGP_ERR_HIP;                                                                  \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, stream, p);                                              \
    }
    if (npairs <= 12) SDGP_NARROW_MM(3)   // few accumulators: three workgroups share a CU
    else SDGP_NARROW_MM(kMmMaxPairs)
#undef SDGP_NARROW_MM
    return launch_status();
}

template <int M, bool NLE2>
int launch_narrow_rk(const NarrowParams& p, int rk, int nt, int grid, int lds, hipStream_t stream) {
    if (nt > 0) {
        if (rk == kRandom) return launch_narrow_mm<M, kRandom, true, NLE2>(p, grid, stream);
        if (rk == kGreedy) return launch_narrow_mm<M, kGreedy, true, NLE2>(p, grid, stream);
        return launch_narrow_mm<M, kAdjusted, true, NLE2>(p, grid, stream);
    }
#define SDGP_NARROW(RKV)                                                                                              \
    {                                                                                                                 \
        auto kern = bwd_narrow<M, RKV, true, NLE2>;                                                                   \
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                       \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);   \
        if (attr != hipSuccess) return SDGP_ERR_HIP;                                                                  \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, stream, p);                                              \
    }
    if (rk == kRandom) SDGP_NARROW(kRandom)
    else if (rk == kGreedy) SDGP_NARROW(kGreedy)
    else SDGP_NARROW(kAdjusted)
#undef SDGP_NARROW
    return launch_status();
}

}  // namespace

namespace {

// The tiling of a problem; SDGP_OK, or a positive value when this file's kernels do not take it.  nt (p.nt) is the
// matrix-core variant's column tiles, 0 for the vector-ALU variant; lds is the latter's LDS size.
int narrow_plan(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n, int m,
                NarrowParams& p, int64_t& grid, int& lds) {
    if (C_in < 1 || C_in > 4 || (C_out % 8) != 0) return 1;
    if (n != m && !(m == 4 || m == 8 || m == 16)) return 1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    if (B * P * Q >= INT32_MAX || B * H * Wd >= INT32_MAX) return 1;
    p.B = (int)B, p.H = (int)H, p.Wd = (int)Wd, p.P = (int)P, p.Q = (int)Q, p.C_in = (int)C_in, p.C_out = (int)C_out;
    p.R = R, p.S = S, p.stride = stride, p.pad = pad, p.n = n;
    p.TW = (int)(Wd < 16 ? Wd : 16);
    p.TH = (int)(H < 256 / p.TW ? H : 256 / p.TW);
    p.tiles_h = ((int)H + p.TH - 1) / p.TH, p.tiles_w = ((int)Wd + p.TW - 1) / p.TW;
    // gradient rows (columns) a tile's taps can reach: those whose multiple of the stride falls into a span of TH + R - 1
    p.HP = (p.TH - 1 + R - 1) / stride + 1, p.HQ = (p.TW - 1 + S - 1) / stride + 1;
    if (p.HQ < 2) p.HQ = 2;  // the reciprocal below needs a divisor above one
    p.hq_magic = (uint32_t)((1ull << 32) / (uint64_t)p.HQ) + 1u;
    grid = (int64_t)B * p.tiles_h * p.tiles_w;
    if (grid >= INT32_MAX) return 1;
    // the matrix-core variant when its (row tile, column tile) pairs and LDS fit; else the vector-ALU one
    const int J = R * S * (int)C_in, npix = p.HP * p.HQ;
    int nt = (J + 31) / 32;
    if (nt > kMmMaxNt || ((npix + 31) / 32) * nt > 4 * kMmMaxPairs || narrow_mm_lds(npix, nt, J) > 160 * 1024) nt = 0;
    p.nt = nt;
    p.nt_magic = nt > 0 ? (uint32_t)(65536 / nt + 1) : 0u;
    lds = ((npix * kAPitchN + 15) & ~15) + kNarrowKC * R * S * 16;
    if (nt == 0 && lds > 160 * 1024) return 1;
    return SDGP_OK;
}

// Bytes of the filter image for a planned problem: worth building when the filter slice is more than one column tile
// (the 7x7 stem: 160 columns; a 3x3 filter on three channels fits one tile and is gathered inside the kernel).
size_t narrow_image_bytes(const NarrowParams& p) {
    if (p.nt < 2) return 0;
    const size_t slices = (size_t)((p.C_out + kNarrowKC - 1) / kNarrowKC);
    return slices * (size_t)narrow_image_units(p.nt) * 1024u;
}

}  // namespace

// Workspace bytes bwd_narrow_launch wants for these arguments (0: none, also when another kernel takes the problem).
size_t bwd_narrow_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride,
                            int pad, int n, int m) {
    NarrowParams p{};
    int64_t grid = 0;
    int lds = 0;
    if (narrow_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, p, grid, lds) != SDGP_OK || grid == 0) return 0;
    const size_t image = narrow_image_bytes(p);
    if (first2_fits(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m) && first2_image_bytes(C_out) > image) return first2_image_bytes(C_out);
    return image;
}

// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.  workspace:
// bwd_narrow_workspace(...) bytes, 16-byte aligned, or null (the kernel then gathers the filter itself).
int bwd_narrow_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                      int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                      void* workspace, hipStream_t stream) {
    if (!is_aligned16(dO)) return 1;
    if (stream_fits(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m)) {
        StreamParams f{};
        f.dO = static_cast<const uint16_t*>(dO), f.W = static_cast<const uint16_t*>(W), f.dD = static_cast<uint16_t*>(dD);
        f.B = (int)B, f.H = (int)H, f.Wd = (int)Wd, f.C_in = (int)C_in;
        f.strips = (int)((Wd + 31) / 32);
        // one wavefront per (image, strip, range of block rows): about 1024 of them (four per CU) when the batch allows,
        // ranges of at least four block rows
        const int64_t units = B * f.strips, rows = H / 2;
        int64_t splits = units >= 1024 ? 1 : (1024 + units - 1) / units;
        if (splits > rows / 4) splits = rows / 4 > 0 ? rows / 4 : 1;
        f.steps_per_split = (int)((rows + splits - 1) / splits);
        f.splits = (int)((rows + f.steps_per_split - 1) / f.steps_per_split);
        f.tasks = (int)(units * f.splits);
        f.n = n, f.mix = seed_mix(seed);
        if (n == m) return launch_stream<4, kGreedy, false, true>(f, stream);
        const bool le2 = n <= 2;
        if (m == 4) return le2 ? launch_stream_rk<4, true>(f, rk, stream) : launch_stream_rk<4, false>(f, rk, stream);
        if (m == 8) return le2 ? launch_stream_rk<8, true>(f, rk, stream) : launch_stream_rk<8, false>(f, rk, stream);
        return le2 ? launch_stream_rk<16, true>(f, rk, stream) : launch_stream_rk<16, false>(f, rk, stream);
    }
    // (measured on the ImageNet stem at batch 256: 153 us against the tile kernel's 188 us dense, but 296 against 270 us
    // with 2:4 pruning -- a block row per step reads every gradient fragment from LDS for one matrix instruction only,
    // and the in-place ranking of one 19-pixel row fills its wavefront poorly -- so only the dense product streams)
    if (n == m && stem_stream_fits(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m)) {
        StemStreamParams f{};
        f.dO = static_cast<const uint16_t*>(dO), f.W = static_cast<const uint16_t*>(W), f.dD = static_cast<uint16_t*>(dD);
        f.B = (int)B, f.P = (int)(H / 2), f.Q = (int)(Wd / 2), f.C_in = (int)C_in;
        f.strips = (f.Q + 15) / 16;
        // one wavefront per (image, strip, range of block rows): about 2048 of them (eight per CU) when the batch allows,
        // ranges of at least eight block rows
        const int64_t units = B * f.strips, rows = f.P;
        int64_t splits = units >= 2048 ? 1 : (2048 + units - 1) / units;
        if (splits > rows / 8) splits = rows / 8 > 0 ? rows / 8 : 1;
        f.steps_per_split = (int)((rows + splits - 1) / splits);
        f.splits = (int)((rows + f.steps_per_split - 1) / f.steps_per_split);
        f.tasks = (int)(units * f.splits);
        f.n = n, f.mix = seed_mix(seed);
        return launch_stem_stream<4, kGreedy, false, true>(f, stream);
    }
    if (workspace != nullptr && is_aligned16(workspace) && B * H * Wd > 0 && first2_fits(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m)) {
        FirstParams f{};
        f.dO = static_cast<const uint16_t*>(dO), f.vimg = static_cast<const unsigned char*>(workspace), f.dD = static_cast<uint16_t*>(dD);
        f.B = (int)B, f.P = (int)(H / 2), f.Q = (int)(Wd / 2), f.C_in = (int)C_in, f.C_out = (int)C_out;
        f.tiles_i = (f.P + kFRows - 1) / kFRows, f.tiles_j = (f.Q + kFCols - 1) / kFCols;
        f.n = n, f.mix = seed_mix(seed);
        hipLaunchKernelGGL(first_v_image, dim3((unsigned)(C_out / kFKC * 16)), dim3(256), 0, stream, static_cast<const uint16_t*>(W),
                           static_cast<uint16_t*>(workspace), (int)C_in);
        if (n == m) return launch_first2<4, kGreedy, false, true>(f, stream);
        const bool le2 = n <= 2;
        if (m == 4) return le2 ? launch_first2_rk<4, true>(f, rk, stream) : launch_first2_rk<4, false>(f, rk, stream);
        if (m == 8) return le2 ? launch_first2_rk<8, true>(f, rk, stream) : launch_first2_rk<8, false>(f, rk, stream);
        return le2 ? launch_first2_rk<16, true>(f, rk, stream) : launch_first2_rk<16, false>(f, rk, stream);
    }
    NarrowParams p{};
    int64_t grid = 0;
    int lds = 0;
    if (narrow_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, p, grid, lds) != SDGP_OK) return 1;
    p.dO = static_cast<const uint16_t*>(dO), p.W = static_cast<const uint16_t*>(W), p.dD = static_cast<uint16_t*>(dD);
    p.mix = seed_mix(seed);
    if (grid == 0) return SDGP_OK;
    const bool dense = n == m;
    const int nt = p.nt;
    const size_t image = narrow_image_bytes(p);
    if (image > 0 && workspace != nullptr && is_aligned16(workspace)) {
        p.wimg = static_cast<const unsigned char*>(workspace);
        p.wimg_units = narrow_image_units(nt);
        const int slices = (p.C_out + kNarrowKC - 1) / kNarrowKC;
        hipLaunchKernelGGL(narrow_w_image, dim3(slices), dim3(256), 0, stream, p.W, static_cast<uint16_t*>(workspace), p.C_out,
                           R * S * p.C_in, p.wimg_units);
    }
    if (dense && nt > 0) return launch_narrow_mm<4, kGreedy, false, true>(p, (int)grid, stream);
    if (dense) {
        auto kern = bwd_narrow<4, kGreedy, false, true>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return SDGP_ERR_HIP;
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, stream, p);
        return launch_status();
    }
    const bool nle2 = n <= 2;
    if (m == 4) return nle2 ? launch_narrow_rk<4, true>(p, rk, nt, (int)grid, lds, stream) : launch_narrow_rk<4, false>(p, rk, nt, (int)grid, lds, stream);
    if (m == 8) return nle2 ? launch_narrow_rk<8, true>(p, rk, nt, (int)grid, lds, stream) : launch_narrow_rk<8, false>(p, rk, nt, (int)grid, lds, stream);
    return nle2 ? launch_narrow_rk<16, true>(p, rk, nt, (int)grid, lds, stream) : launch_narrow_rk<16, false>(p, rk, nt, (int)grid, lds, stream);
}

}  // namespace sdgp
