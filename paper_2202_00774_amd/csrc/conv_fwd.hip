// Forward convolution (Sec. II-A, Fig. 1): O[b,p,q,k] = sum_{r,s,c} D[b, p*stride + r - pad, q*stride + s - pad, c] * W[k,r,s,c].
//
// With stride 1 and a square filter this is the backward-data sum of the mirrored, transposed filter
//   V[c, r', s', k] = W[k, R-1-r', S-1-s', c]   with padding R-1-pad,
// read with the roles of the two channel axes exchanged, so the dense (n == m) matrix-core kernels of the backward-data
// path compute it; this file holds the kernel that builds V and the shape-agnostic kernel (any stride, any filter) for
// the layers that identity does not cover.  The forward pass prunes nothing.
#include "common.h"

namespace sdgp {

namespace {

constexpr int kBlock = 256;

// V[c][r][s][k] = W[k][R-1-r][S-1-s][c]; one thread per element of V, consecutive threads along k.
template <typename T>
__global__ void __launch_bounds__(kBlock) mirror_transpose_filter(const T* W, T* V, int64_t C_out, int64_t C_in, int R, int S) {
    const int64_t total = C_out * C_in * R * S;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int64_t k = i % C_out;
    const int s = (int)((i / C_out) % S);
    const int r = (int)((i / (C_out * S)) % R);
    const int64_t c = i / (C_out * S * R);
    V[i] = W[((k * R + (R - 1 - r)) * S + (S - 1 - s)) * C_in + c];
}

struct FwdArgs {
    const void* D;
    const void* W;
    void* O;
    int64_t B, H, Wd, P, Q, C_in, C_out;
    int R, S, stride, pad;
};

// One thread per element of O; fp32 accumulation over taps, then channels.
template <int DT>
__global__ void __launch_bounds__(kBlock) fwd_simple(FwdArgs a) {
    const int64_t total = a.B * a.P * a.Q * a.C_out;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int64_t k = i % a.C_out, pix = i / a.C_out;
    const int64_t q = pix % a.Q, p = (pix / a.Q) % a.P, b = pix / (a.Q * a.P);
    float acc = 0.0f;
    for (int r = 0; r < a.R; ++r) {
        const int64_t h = p * a.stride + r - a.pad;
        if (h < 0 || h >= a.H) continue;
        for (int s = 0; s < a.S; ++s) {
            const int64_t w = q * a.stride + s - a.pad;
            if (w < 0 || w >= a.Wd) continue;
            const int64_t d0 = ((b * a.H + h) * a.Wd + w) * a.C_in, w0 = ((k * a.R + r) * a.S + s) * a.C_in;
            for (int64_t c = 0; c < a.C_in; ++c) {
                float x, v;
                if constexpr (DT == SDGP_BF16) {
                    x = bf16_to_float(reinterpret_cast<const uint16_t*>(a.D)[d0 + c]);
                    v = bf16_to_float(reinterpret_cast<const uint16_t*>(a.W)[w0 + c]);
                } else {
                    x = reinterpret_cast<const float*>(a.D)[d0 + c];
                    v = reinterpret_cast<const float*>(a.W)[w0 + c];
                }
                acc = fmaf(x, v, acc);
            }
        }
    }
    if constexpr (DT == SDGP_BF16) reinterpret_cast<uint16_t*>(a.O)[i] = (uint16_t)float_to_bf16(acc);
    else reinterpret_cast<float*>(a.O)[i] = acc;
}

// Layers with few input channels (a network's first layer: R*S*C_in of 27 or 147): the reduction is too short for
// the matrix cores' tiles, so plain FMAs do it.  A workgroup keeps the whole filter in LDS as fp32 [tap*channel][k] and
// walks over segments of up to 64 pixels of one output row; thread (k = tid % 64, g = tid / 64) computes pixels
// g, g + 4, ... of the segment for output channel k (and k + 64).  The R image rows a segment touches sit in LDS as
// fp32: the patch of a pixel is a contiguous run of each, and every lane of a wavefront reads the same patch element.
constexpr int kNarrowMaxT = 256;      // R * S * C_in
constexpr int kNarrowGroups = 2048;   // workgroups of a launch (each walks over several segments)

struct NarrowFwdArgs {
    const uint16_t* D;
    const uint16_t* W;
    uint16_t* O;
    int64_t B, segments;              // segments = B * P * ceil(Q / 64)
    int H, Wd, P, Q, C_in, C_out, R, S, stride, pad;
    int T, SC, rowlen, qsegs;         // R*S*C_in, S*C_in, values per staged image row, segments per output row
    uint32_t cin_magic;               // ceil(2^16 / C_in): x / C_in == (x * magic) >> 16 for the x of a staged row
};

template <int KB, int NPT>   // KB = C_out / 64: 1 or 2; NPT pixels per thread, 4 * NPT per segment
__global__ void __launch_bounds__(kBlock) fwd_narrow(NarrowFwdArgs a) {
    constexpr int kNarrowPix = 4 * NPT, kNarrowPerThread = NPT;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* const wl = lds;                                   // [T][64 * KB]
    float* const halo = lds + a.T * 64 * KB;                 // [R][rowlen]
    const int tid = threadIdx.x, k = tid & 63, g = tid >> 6;
    for (int e = tid; e < a.T * 64 * KB; e += kBlock) {
        const int kk = e % (64 * KB), t = e / (64 * KB);
        wl[e] = bf16_to_float(a.W[(int64_t)kk * a.T + t]);
    }
    for (int64_t seg = blockIdx.x; seg < a.segments; seg += gridDim.x) {
        const int q0 = (int)(seg % a.qsegs) * kNarrowPix;
        const int p = (int)((seg / a.qsegs) % a.P);
        const int64_t b = seg / ((int64_t)a.qsegs * a.P);
        const int npx = a.Q - q0 < kNarrowPix ? a.Q - q0 : kNarrowPix;
        __syncthreads();   // the previous segment's rows have been read (and, the first time, the filter is staged)
        for (int r = 0; r < a.R; ++r) {
            const int h = p * a.stride + r - a.pad;
            const uint16_t* const src = a.D + ((b * a.H + h) * (int64_t)a.Wd + q0 * a.stride - a.pad) * a.C_in;
            for (int x = tid; x < a.rowlen; x += kBlock) {
                const int w = q0 * a.stride - a.pad + (int)(((uint32_t)x * a.cin_magic) >> 16);
                halo[r * a.rowlen + x] = (h >= 0 && h < a.H && w >= 0 && w < a.Wd) ? bf16_to_float(src[x]) : 0.0f;
            }
        }
        __syncthreads();
        float acc[KB][kNarrowPerThread];
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
            for (int j = 0; j < kNarrowPerThread; ++j) acc[u][j] = 0.0f;
        for (int r = 0; r < a.R; ++r) {
            const float* const row = halo + r * a.rowlen + g * a.stride * a.C_in;
            const float* const wr = wl + (r * a.SC) * 64 * KB + k;
            for (int t = 0; t < a.SC; ++t) {
                float wv[KB];
#pragma unroll
                for (int u = 0; u < KB; ++u) wv[u] = wr[t * 64 * KB + u * 64];
#pragma unroll
                for (int j = 0; j < kNarrowPerThread; ++j) {
                    const float xv = row[j * 4 * a.stride * a.C_in + t];   // pixels past the segment's end: computed, not stored
#pragma unroll
                    for (int u = 0; u < KB; ++u) acc[u][j] = fmaf(xv, wv[u], acc[u][j]);
                }
            }
        }
        uint16_t* const out = a.O + ((b * a.P + p) * (int64_t)a.Q + q0) * a.C_out + k;
#pragma unroll
        for (int j = 0; j < kNarrowPerThread; ++j) {
            const int px = g + 4 * j;
            if (px < npx) {
#pragma unroll
                for (int u = 0; u < KB; ++u) out[(int64_t)px * a.C_out + u * 64] = (uint16_t)float_to_bf16(acc[u][j]);
            }
        }
    }
}

}  // namespace

int mirror_transpose_filter_launch(const void* W, void* V, int64_t C_out, int64_t C_in, int R, int S, int dt,
                                   hipStream_t stream) {
    const int64_t total = C_out * C_in * R * S;
    if (total == 0) return SDGP_OK;
    const int64_t blocks = (total + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFF) return SDGP_ERR_SHAPE;
    if (dt == SDGP_BF16)
        mirror_transpose_filter<uint16_t><<<(unsigned)blocks, kBlock, 0, stream>>>((const uint16_t*)W, (uint16_t*)V, C_out, C_in, R, S);
    else
        mirror_transpose_filter<uint32_t><<<(unsigned)blocks, kBlock, 0, stream>>>((const uint32_t*)W, (uint32_t*)V, C_out, C_in, R, S);
    return launch_status();
}

int fwd_simple_launch(const void* D, const void* W, void* O, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                      int R, int S, int stride, int pad, int dt, hipStream_t stream) {
    FwdArgs a{D, W, O, B, H, Wd, (H + 2 * pad - R) / stride + 1, (Wd + 2 * pad - S) / stride + 1, C_in, C_out, R, S, stride, pad};
    const int64_t total = a.B * a.P * a.Q * a.C_out;
    if (total == 0) return SDGP_OK;
    const int64_t blocks = (total + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFF) return SDGP_ERR_SHAPE;
    if (dt == SDGP_BF16) fwd_simple<SDGP_BF16><<<(unsigned)blocks, kBlock, 0, stream>>>(a);
    else fwd_simple<SDGP_F32><<<(unsigned)blocks, kBlock, 0, stream>>>(a);
    return launch_status();
}

}  // namespace sdgp

namespace sdgp {

// bf16 layers with R*S*C_in <= 256 and 64 or 128 output channels; 1 when the layer is not of that kind.
int fwd_narrow_launch(const void* D, const void* W, void* O, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                      int R, int S, int stride, int pad, int dt, hipStream_t stream) {
    const int64_t T = (int64_t)R * S * C_in;
    if (dt != SDGP_BF16 || T > kNarrowMaxT || (C_out != 64 && C_out != 128) || C_in >= 32) return 1;
    if (H > (1 << 24) || Wd > (1 << 24)) return 1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    NarrowFwdArgs a{};
    a.D = (const uint16_t*)D, a.W = (const uint16_t*)W, a.O = (uint16_t*)O, a.B = B;
    a.H = (int)H, a.Wd = (int)Wd, a.P = (int)P, a.Q = (int)Q, a.C_in = (int)C_in, a.C_out = (int)C_out;
    a.R = R, a.S = S, a.stride = stride, a.pad = pad;
    a.T = (int)T, a.SC = S * (int)C_in;
    const int pix = Q <= 32 ? 32 : 64;   // pixels per segment
    a.rowlen = ((pix - 1) * stride + S) * (int)C_in;
    a.qsegs = (int)((Q + pix - 1) / pix);
    a.segments = B * P * a.qsegs;
    a.cin_magic = (65536u + (uint32_t)C_in - 1) / (uint32_t)C_in;
    if (a.segments == 0) return SDGP_OK;
    const size_t lds = ((size_t)T * C_out + (size_t)R * a.rowlen) * sizeof(float);
    if (lds > 150 * 1024 || a.rowlen > 2048) return 1;
    const unsigned grid = (unsigned)(a.segments < kNarrowGroups ? a.segments : kNarrowGroups);
    void (*kernel)(NarrowFwdArgs) = C_out == 64 ? (pix == 32 ? fwd_narrow<1, 8> : fwd_narrow<1, 16>)
                                                : (pix == 32 ? fwd_narrow<2, 8> : fwd_narrow<2, 16>);
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SDGP_ERR_HIP;
    kernel<<<grid, kBlock, lds, stream>>>(a);
    return launch_status();
}

}  // namespace sdgp
