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
