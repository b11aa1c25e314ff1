// Simple fused backward-data kernel: one thread per element of dL/dD.
//
// This is the shape-agnostic path (any dtype, any 1 <= n <= m <= 32, any
// filter, stride and padding, channel counts that are not multiples of the
// vector width).  Every thread walks the taps that reach its input pixel
// (Fig. 3 left), prunes each group of the gradient row it meets with the
// pruning function of Sec. III-B, and accumulates kept * W in fp32.  Ranking is
// repeated by every thread that needs the group; the tiled MFMA kernels exist
// to avoid exactly that, this one is for shapes they do not take.
#include "ranker.h"

namespace sdgp {

namespace {

constexpr int kBlock = 256;

struct SimpleArgs {
    const void* dO;
    const void* W;
    void* dD;
    int64_t B, H, Wd, P, Q, C_in, C_out;
    int R, S, stride, pad;
    int n, m, rk;
    uint32_t mix;
    int64_t cig, cog;   // channels per convolution group (all of them when there is one group)
};

template <int DT>
__device__ __forceinline__ uint32_t load_raw(const void* p, int64_t i) {
    if constexpr (DT == kBF16) return (uint32_t) reinterpret_cast<const uint16_t*>(p)[i];
    else return reinterpret_cast<const uint32_t*>(p)[i];
}

template <int DT>
__device__ __forceinline__ float raw_to_float(uint32_t r) {
    if constexpr (DT == kBF16) return bf16_to_float(r);
    else return bits_to_float(r);
}

// Pruned values (as fp32) of the m-group starting at flat element e0.
template <int DT>
__device__ void pruned_group(const void* dO, uint64_t e0, int n, int m, int rk, uint32_t mix, float* val) {
    constexpr uint32_t kMagMask = (DT == kBF16) ? 0x7FFFu : 0x7FFFFFFFu;
    uint32_t raw[32], key[32];
    for (int j = 0; j < m; ++j) {
        raw[j] = load_raw<DT>(dO, (int64_t)e0 + j);
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
            const float a = bits_to_float(float_to_bits(raw_to_float<DT>(raw[j])) & 0x7FFFFFFFu);
            total = __fadd_rn(total, a);
            if ((keepmask >> j) & 1u) kept = __fadd_rn(kept, a);
        }
        scale = (kept == 0.0f) ? 1.0f : __fdiv_rn(total, kept);
    }
    for (int j = 0; j < m; ++j) {
        float y = 0.0f;
        if ((keepmask >> j) & 1u) {
            y = raw_to_float<DT>(raw[j]);
            if (rk == kAdjusted) {
                y = __fmul_rn(y, scale);
                if constexpr (DT == kBF16) y = bf16_to_float(float_to_bf16(y));  // the pruned tensor is stored in bf16
            }
        }
        val[j] = y;
    }
}

template <int DT>
__global__ void __launch_bounds__(kBlock) bwd_simple(SimpleArgs a) {
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t total = a.B * a.H * a.Wd * a.C_in;
    if (t >= total) return;
    const int64_t c = t % a.C_in;
    const int64_t pix = t / a.C_in;
    const int64_t w = pix % a.Wd, h = (pix / a.Wd) % a.H, b = pix / (a.Wd * a.H);

    const int64_t g = c / a.cig, cl = c - g * a.cig;   // the convolution group of this input channel
    float acc = 0.0f;
    for (int r = 0; r < a.R; ++r) {
        const int64_t hp = h + a.pad - r;
        if (hp < 0 || hp % a.stride != 0) continue;
        const int64_t p = hp / a.stride;
        if (p >= a.P) continue;
        for (int s = 0; s < a.S; ++s) {
            const int64_t wq = w + a.pad - s;
            if (wq < 0 || wq % a.stride != 0) continue;
            const int64_t q = wq / a.stride;
            if (q >= a.Q) continue;
            const uint64_t row0 = (uint64_t)((b * a.P + p) * a.Q + q) * (uint64_t)a.C_out;
            for (int64_t k0 = g * a.cog; k0 < (g + 1) * a.cog; k0 += a.m) {
                float val[32];
                if (a.n == a.m) {
                    for (int j = 0; j < a.m; ++j) val[j] = raw_to_float<DT>(load_raw<DT>(a.dO, (int64_t)row0 + k0 + j));
                } else {
                    pruned_group<DT>(a.dO, row0 + (uint64_t)k0, a.n, a.m, a.rk, a.mix, val);
                }
                for (int j = 0; j < a.m; ++j) {
                    const float wv = raw_to_float<DT>(load_raw<DT>(a.W, (((k0 + j) * a.R + r) * a.S + s) * a.cig + cl));
                    acc = fmaf(val[j], wv, acc);
                }
            }
        }
    }
    if constexpr (DT == kBF16) reinterpret_cast<uint16_t*>(a.dD)[t] = (uint16_t)float_to_bf16(acc);
    else reinterpret_cast<float*>(a.dD)[t] = acc;
}

}  // namespace

// groups > 1: W is [C_out, R, S, C_in / groups] and input channel c sums over the output channels of its group only
// (C_in and C_out multiples of groups, C_out / groups a multiple of m: the callers check).
int bwd_simple_grouped_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                              int64_t C_out, int R, int S, int stride, int pad, int64_t groups, int dt, int n, int m, int rk,
                              uint64_t seed, hipStream_t stream) {
    SimpleArgs a;
    a.cig = C_in / groups, a.cog = C_out / groups;
    a.dO = dO, a.W = W, a.dD = dD;
    a.B = B, a.H = H, a.Wd = Wd, a.C_in = C_in, a.C_out = C_out;
    a.P = (H + 2 * pad - R) / stride + 1, a.Q = (Wd + 2 * pad - S) / stride + 1;
    a.R = R, a.S = S, a.stride = stride, a.pad = pad, a.n = n, a.m = m, a.rk = rk, a.mix = seed_mix(seed);
    const int64_t total = B * H * Wd * C_in;
    if (total == 0) return SDGP_OK;
    const dim3 grid((unsigned)((total + kBlock - 1) / kBlock)), block(kBlock);
    if (dt == kBF16) hipLaunchKernelGGL(bwd_simple<kBF16>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(bwd_simple<kF32>, grid, block, 0, stream, a);
    return launch_status();
}

int bwd_simple_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                      int64_t C_out, int R, int S, int stride, int pad, int dt, int n, int m, int rk, uint64_t seed,
                      hipStream_t stream) {
    return bwd_simple_grouped_launch(dO, W, dD, B, H, Wd, C_in, C_out, R, S, stride, pad, 1, dt, n, m, rk, seed, stream);
}

}  // namespace sdgp
