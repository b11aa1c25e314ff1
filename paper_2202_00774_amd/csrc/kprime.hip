// Backward-data product from the COMPACTED gradient: K' = (n/m) * C_out kept values per pixel, each with the position
// of its channel, and the matching rows of W gathered by that index (Sec. III-A: "2 multiplications instead of 4";
// Sec. IV-C: the ratio-4 and ratio-8 estimates assume work proportional to n/m).
//
// Every pixel keeps different channels, so the gathered rows differ from pixel to pixel and the product is not a
// matrix product: it is one AXPY per kept value,
//   dD[b,h,w,:] += v * W[k, r, s, :]        for every tap (r,s) that reaches (h,w) and every kept (v, k) of its pixel,
// done here with fp32 FMAs on the vector ALUs.  Its work falls with n/m where the structured-sparse matrix instruction's
// stays at one half, so it can only win at high sparsity; the benchmark measures where.
//
//   * input: the compact output of the prune pass (values [pixels][K'] in bf16, positions [pixels][K'] as bytes);
//   * a workgroup takes a run of output pixels and a block of CB = 8 * LPP input channels; a pixel is served by LPP
//     lanes holding 8 channels each (one 16-byte LDS read of a W row per kept value), a wavefront covers 64 / LPP
//     pixels at a time and 8 such passes: 64 fp32 accumulators per lane;
//   * W travels through LDS in chunks of KC output channels (all taps, the block's channels), a multiple of m, so
//     the entries of a pixel that belong to a chunk are a contiguous run of its compact row.
#include "common.h"

namespace sdgp {

namespace {

constexpr int kThreads = 256;
constexpr int kPasses = 8;
constexpr int kChunkBytes = 64 * 1024;

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

struct KprimeArgs {
    const uint16_t* vals;   // [B*P*Q][Kp]
    const uint8_t* idx;     // [B*P*Q][Kp], position inside the group of m
    const uint16_t* W;      // [C_out][R][S][C_in]
    uint16_t* dD;           // [B][H][Wd][C_in]
    int64_t npix;           // B * H * Wd
    int H, Wd, P, Q, C_in, C_out, R, S, stride, pad, n, m;
    int Kp, KC, cblocks, pix_per_wg;
    int nshift;             // log2(n) when n is a power of two, else -1
    int vec4;               // every (pixel, chunk) run of entries starts at a multiple of 4 and has a multiple of 4 entries
};

template <int LPP>
__global__ void __launch_bounds__(kThreads) kprime_axpy(KprimeArgs a) {
    constexpr int CB = 8 * LPP, PPW = 64 / LPP;
    extern __shared__ __attribute__((aligned(16))) unsigned char wl[];   // [KC][taps][CB] bf16
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPP, grp = lane / LPP;
    const int cb = blockIdx.x % a.cblocks;
    const int64_t pix0 = (int64_t)(blockIdx.x / a.cblocks) * a.pix_per_wg + wave * (PPW * kPasses);
    const int taps = a.R * a.S;
    const int c0 = cb * CB + sub * 8;

    float acc[kPasses][8];
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[ps][e] = 0.0f;

    // the output pixel of each pass: image and coordinates (-1 when past the tensor's end)
    int ph[kPasses], pw[kPasses];
    int64_t pb[kPasses];
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
        const int64_t pix = pix0 + ps * PPW + grp;
        const bool live = pix < a.npix;
        pw[ps] = live ? (int)(pix % a.Wd) : -1;
        ph[ps] = live ? (int)((pix / a.Wd) % a.H) : -1;
        pb[ps] = live ? pix / ((int64_t)a.Wd * a.H) : 0;
    }

    for (int k0 = 0; k0 < a.C_out; k0 += a.KC) {
        const int rows = a.C_out - k0 < a.KC ? a.C_out - k0 : a.KC;
        __syncthreads();   // the previous chunk has been read
        for (int u = tid; u < rows * taps * LPP; u += kThreads) {
            const int s16 = u % LPP, rt = u / LPP;          // rt = k_local * taps + tap
            const int c = cb * CB + s16 * 8;
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (c < a.C_in) v = *reinterpret_cast<const u32x4_t*>(a.W + ((int64_t)k0 * taps + rt) * a.C_in + c);
            *reinterpret_cast<u32x4_t*>(wl + (int64_t)u * 16) = v;
        }
        __syncthreads();
        const int e0 = k0 / a.m * a.n, ecount = rows / a.m * a.n;
#pragma unroll
        for (int ps = 0; ps < kPasses; ++ps) {
            if (pw[ps] < 0) continue;
            for (int r = 0; r < a.R; ++r) {
                const int hp = ph[ps] + a.pad - r;
                if (hp < 0 || hp % a.stride != 0 || hp / a.stride >= a.P) continue;
                for (int s = 0; s < a.S; ++s) {
                    const int wq = pw[ps] + a.pad - s;
                    if (wq < 0 || wq % a.stride != 0 || wq / a.stride >= a.Q) continue;
                    const int64_t src = ((pb[ps] * a.P + hp / a.stride) * a.Q + wq / a.stride) * a.Kp + e0;
                    const unsigned char* const wtap = wl + ((r * a.S + s) * LPP + sub) * 16;
                    // four entries at a time: their loads and LDS reads are issued before the first FMA needs them
                    for (int e = 0; e < ecount; e += 4) {
                        float v[4];
                        int kl[4];
                        if (a.vec4) {
                            const uint2 v4 = *reinterpret_cast<const uint2*>(a.vals + src + e);
                            const uint32_t i4 = *reinterpret_cast<const uint32_t*>(a.idx + src + e);
                            v[0] = bits_to_float(v4.x << 16), v[1] = bits_to_float(v4.x & 0xFFFF0000u);
                            v[2] = bits_to_float(v4.y << 16), v[3] = bits_to_float(v4.y & 0xFFFF0000u);
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const int gi = a.nshift >= 0 ? ((e + u) >> a.nshift) : (e + u) / a.n;
                                kl[u] = gi * a.m + (int)((i4 >> (8 * u)) & 0xFFu);
                            }
                        } else {
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const bool live = e + u < ecount;
                                const int ee = live ? e + u : ecount - 1;     // a slot past the run repeats its last entry with value 0
                                v[u] = live ? bf16_to_float(a.vals[src + ee]) : 0.0f;
                                const int gi = a.nshift >= 0 ? (ee >> a.nshift) : ee / a.n;
                                kl[u] = gi * a.m + a.idx[src + ee];
                            }
                        }
                        u32x4_t w8[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) w8[u] = *reinterpret_cast<const u32x4_t*>(wtap + kl[u] * (taps * LPP * 16));
#pragma unroll
                        for (int u = 0; u < 4; ++u)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                acc[ps][2 * j] = fmaf(v[u], bits_to_float(w8[u][j] << 16), acc[ps][2 * j]);
                                acc[ps][2 * j + 1] = fmaf(v[u], bits_to_float(w8[u][j] & 0xFFFF0000u), acc[ps][2 * j + 1]);
                            }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
        if (pw[ps] < 0 || c0 >= a.C_in) continue;
        const int64_t pix = pix0 + ps * PPW + grp;
        u32x4_t o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = float2_to_bf16x2(acc[ps][2 * j], acc[ps][2 * j + 1]);
        *reinterpret_cast<u32x4_t*>(a.dD + pix * a.C_in + c0) = o;
    }
}

}  // namespace

// 0 launched, 1 not taken (C_in not a multiple of 8, or a group of m filter rows does not fit LDS), < 0 error.
int kprime_launch(const void* vals, const uint8_t* idx, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                  int64_t C_out, int R, int S, int stride, int pad, int n, int m, hipStream_t stream) {
    if (C_in % 8 != 0 || C_in == 0 || C_out == 0 || H > (1 << 24) || Wd > (1 << 24) || C_out > (1 << 20)) return 1;
    KprimeArgs a{};
    a.vals = (const uint16_t*)vals, a.idx = idx, a.W = (const uint16_t*)W, a.dD = (uint16_t*)dD;
    a.npix = B * H * Wd;
    a.H = (int)H, a.Wd = (int)Wd, a.P = (int)((H + 2 * pad - R) / stride + 1), a.Q = (int)((Wd + 2 * pad - S) / stride + 1);
    a.C_in = (int)C_in, a.C_out = (int)C_out, a.R = R, a.S = S, a.stride = stride, a.pad = pad, a.n = n, a.m = m;
    a.Kp = (int)(C_out / m * n);
    const int lpp = C_in <= 64 ? 8 : C_in <= 128 ? 16 : C_in <= 256 ? 32 : 64;
    const int cbytes = lpp * 16, taps = R * S;
    int kc = kChunkBytes / (taps * cbytes) / m * m;
    if (kc < m) kc = m;
    if ((int64_t)kc * taps * cbytes > 150 * 1024) return 1;
    if (kc > C_out) kc = (int)C_out;
    a.KC = kc;
    a.nshift = (n & (n - 1)) == 0 ? __builtin_ctz((unsigned)n) : -1;
    a.vec4 = (a.Kp % 4 == 0 && (kc / m * n) % 4 == 0) ? 1 : 0;
    a.cblocks = (int)((C_in + lpp * 8 - 1) / (lpp * 8));
    a.pix_per_wg = 4 * (64 / lpp) * kPasses;
    const int64_t blocks = ((a.npix + a.pix_per_wg - 1) / a.pix_per_wg) * a.cblocks;
    if (blocks == 0) return SDGP_OK;
    if (blocks > 0x7FFFFFFF) return SDGP_ERR_SHAPE;
    const size_t lds = (size_t)kc * taps * cbytes;
    void (*kernel)(KprimeArgs) = lpp == 8 ? kprime_axpy<8> : lpp == 16 ? kprime_axpy<16> : lpp == 32 ? kprime_axpy<32> : kprime_axpy<64>;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SDGP_ERR_HIP;
    kernel<<<(unsigned)blocks, kThreads, lds, stream>>>(a);
    return launch_status();
}

}  // namespace sdgp
