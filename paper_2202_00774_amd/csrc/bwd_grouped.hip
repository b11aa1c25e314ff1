// Backward-data of a grouped 3x3 convolution with 16 channels per group on both sides (the group width of RegNetX-400MF,
// Sec. IV), stride 1 or 2, padding 1, bf16.  A group is a tiny product -- 16 input channels, reduction over 9 taps x 16
// output channels -- so the matrix instruction is the 16-column one: for one group and 16 consecutive input pixels,
//   dD[c][pixel] = sum_{tap, k} W[k][tap][c] * prune(dO)[pixel + 1 - tap][k],
// with two taps (32 reduction elements) per v_mfma_f32_16x16x32_bf16: five instructions per group and 16 pixels,
// the last one half empty.  A lane ends up with four channels of one input pixel.
//   * workgroup = 4 wavefronts, tile = 8 x 32 input pixels of one image and a slab of four groups (64 channels,
//     128 bytes per pixel); the 10 x 34 gradient pixels the taps reach arrive by direct-to-LDS copies (144-byte
//     pitch: sixteen consecutive pixels read conflict-free), slots outside the image or the tensor's channels are
//     cleared and skipped, every 16-channel item is pruned in place (Alg. 1 runs along all of C_out; with m <= 16 a
//     group of m lies inside one item);
//   * the filter, re-indexed so that a lane's fragment is 16 contiguous bytes ([group][tap pair][c][2 taps x 16 k]),
//     is built once per call in the workspace and goes straight to registers (20 fragments per wavefront);
//   * one pass: a group's whole reduction is in the tile, so there is no loop over chunks;
//   * stride 2: the input pixels split into four parity classes (h mod 2, w mod 2) with 1, 2, 2 and 4 taps -- again five
//     tap pairs.  The tile is 8 x 32 positions (i, j) of the class grid, input pixels (2i + a, 2j + b), all four
//     classes from one gradient tile of 9 x 33 pixels: tap r of class a reads gradient row i + (a + 1 - r) / 2.
#include "lds_copy.h"

namespace sdgp {

namespace {

constexpr int kGW = 16;                                  // channels per group, both sides
constexpr int kGSlab = 4;                                // groups per workgroup
constexpr int kGTH = 8, kGTW = 32;                       // tile, positions of the (class) grid
constexpr int kGPitch = kGSlab * kGW * 2 + 16;           // 144 bytes per pixel in LDS
constexpr int kGSlots = kGPitch / 16;                    // 9 sixteen-byte slots, the last one padding
constexpr int kGPairs = 5;                               // tap pairs
constexpr int kGImageBytes = kGPairs * 16 * 64;          // filter image per group: [pair][c][32] bf16

// Geometry per stride.  kOrigin: the tile's gradient pixels start kOrigin before its first grid position.
template <int STRIDE>
struct GroupedGeom {
    static constexpr int kOrigin = STRIDE == 1 ? 1 : 0;
    static constexpr int kHaloRows = kGTH + (STRIDE == 1 ? 2 : 1), kHaloCols = kGTW + (STRIDE == 1 ? 2 : 1);
    static constexpr int kPix = kHaloRows * kHaloCols;                   // 340 or 297 gradient pixels
    static constexpr int kUnits = (kPix * kGPitch + 1023) / 1024;        // 48 or 42 copy units of 1 KB
    static constexpr int kLds = kUnits * 1024;
    static constexpr uint32_t kColMagic = 65536u / kHaloCols + 1u;       // x / kHaloCols == (x * magic) >> 16 for x < 342
    static constexpr int kClasses = STRIDE * STRIDE;
};
// Tap `which` (0, 1) of pair j as r * 3 + s, or -1: stride 1 pairs the taps in order; stride 2 pairs them inside a
// parity class -- (0,0): the centre; (0,1): (1,0) (1,2); (1,0): (0,1) (2,1); (1,1): (0,0) (0,2) and (2,0) (2,2).
__host__ __device__ constexpr int pair_tap(int stride, int j, int which) {
    if (stride == 1) return 2 * j + which < 9 ? 2 * j + which : -1;
    constexpr int table[kGPairs][2] = {{4, -1}, {3, 5}, {1, 7}, {0, 2}, {6, 8}};
    return table[j][which];
}
__host__ __device__ constexpr int pair_class(int stride, int j) { return stride == 1 ? 0 : (j < 3 ? j : 3); }  // class = 2 a + b
// Gradient row (column) of tap coordinate r for class parity a, relative to the grid position, plus kOrigin.
__host__ __device__ constexpr int tap_shift(int stride, int a, int r) { return stride == 1 ? 2 - r : (a + 1 - r) / 2; }

typedef float f32x4g __attribute__((ext_vector_type(4)));
#define SDGP_LDSG __attribute__((address_space(3)))

struct GroupedParams {
    const uint16_t* dO;
    const unsigned char* wimg;   // [groups][kGPairs][16 c][32] bf16
    uint16_t* dD;
    int B, H, Wd, P, Q, C, groups;   // H x Wd input pixels, P x Q gradient pixels
    int tiles_h, tiles_w, slabs;
    int n;
    uint32_t mix;
};

// One workgroup per (group, tap pair): row c holds W[g*16 + k][tap][c] for tap = 2 pair + (kk >> 4), k = kk & 15.
__global__ void __launch_bounds__(256) grouped_w_image(const uint16_t* __restrict__ W, uint16_t* __restrict__ img, int stride) {
    const int g = blockIdx.x / kGPairs, pair = blockIdx.x % kGPairs;
    uint16_t* dst = img + ((size_t)g * kGPairs + pair) * 512;
    for (int e = threadIdx.x; e < 512; e += 256) {
        const int kk = e & 31, c = e >> 5;
        const int tap = pair_tap(stride, pair, kk >> 4), k = kk & 15;
        dst[e] = tap >= 0 ? W[((size_t)(g * kGW + k) * 9 + tap) * kGW + c] : (uint16_t)0;
    }
}

template <int STRIDE, int M, int RK, bool PRUNE, bool NLE2>
__global__ void __launch_bounds__(256, 2) bwd_group16(const GroupedParams p) {
    using G = GroupedGeom<STRIDE>;
    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDSG unsigned char* smem = (SDGP_LDSG unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int t = blockIdx.x;
    const int slab = t % p.slabs;
    t /= p.slabs;
    const int tw = t % p.tiles_w, th = (t / p.tiles_w) % p.tiles_h, b = t / (p.tiles_w * p.tiles_h);
    const int i0 = th * kGTH, j0 = tw * kGTW;           // first grid position of the tile
    const int g0 = slab * kGSlab;                       // first group of the slab
    const int px = lane & 15, oct = lane >> 4;

    // ---- copies: slot -> (gradient pixel, eight channels); what is not there is cleared
    const unsigned char* const image = reinterpret_cast<const unsigned char*>(p.dO + (size_t)b * p.P * p.Q * p.C);
    constexpr int kUnitsPerWave = (G::kUnits + 3) / 4;
#pragma unroll
    for (int x = 0; x < kUnitsPerWave; ++x) {
        const int u = wave + 4 * x;
        if (u < G::kUnits) {
            const int slot = u * 64 + lane;
            const int pix = (int)(((uint32_t)slot * 7282u) >> 16);              // slot / 9 for slot < 3072
            const int part = slot - kGSlots * pix;                              // 0..7 data, 8 padding
            const int hr = (int)(((uint32_t)pix * G::kColMagic) >> 16);         // pix / kHaloCols
            const int gp = i0 - G::kOrigin + hr, gq = j0 - G::kOrigin + (pix - hr * G::kHaloCols);
            const int ch = g0 * kGW + part * 8;
            const bool ok = part < 8 && pix < G::kPix && gp >= 0 && gp < p.P && gq >= 0 && gq < p.Q && ch < p.C;
            if (ok) lds_copy16(image, (uint32_t)((gp * p.Q + gq) * p.C + ch) * 2u, smem_base + (uint32_t)u * 1024u);
            else *(SDGP_LDSG u32x4_t*)(smem + slot * 16) = u32x4_t{0u, 0u, 0u, 0u};
        }
    }
    // ---- the filter's fragments: lane (c = px, k-octet = oct) of (group, tap pair)
    bf16x8_t wf[kGSlab][kGPairs];
#pragma unroll
    for (int g = 0; g < kGSlab; ++g) {
        const int gg = g0 + g < p.groups ? g0 + g : p.groups - 1;           // (a slab past the last group repeats it; never stored)
#pragma unroll
        for (int j = 0; j < kGPairs; ++j)
            wf[g][j] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(p.wimg + ((size_t)(gg * kGPairs + j) * 16 + px) * 64 + oct * 16));
    }
    wait_lds_copies<0>();
    __syncthreads();
    if constexpr (PRUNE) {
        for (int it = tid; it < G::kPix * kGSlab; it += 256) {
            const int pix = it >> 2, g = it & 3;
            const int hr = (int)(((uint32_t)pix * G::kColMagic) >> 16);
            const int gp = i0 - G::kOrigin + hr, gq = j0 - G::kOrigin + (pix - hr * G::kHaloCols);
            if (gp >= 0 && gp < p.P && gq >= 0 && gq < p.Q && g0 + g < p.groups) {
                SDGP_LDSG u32x4_t* rec = (SDGP_LDSG u32x4_t*)(smem + pix * kGPitch + g * 32);
                u32x4_t v[2] = {rec[0], rec[1]};
                const size_t gpix = (size_t)(b * p.P + gp) * p.Q + gq;
                prune16_dense<M, RK, NLE2>(v, p.n, p.mix, (uint64_t)gpix * (uint64_t)p.C + (uint64_t)((g0 + g) * kGW));
                rec[0] = v[0];
                rec[1] = v[1];
            }
        }
        __syncthreads();
    }
    // ---- products: wavefront `wave` owns grid rows 2 wave and 2 wave + 1, both 16-position column groups, four groups.
    // lane's gradient fragment of tap pair j: its tap is the pair's first (oct < 2) or second one; a pair without a
    // second tap reads the first one's pixels against zero weights
    uint32_t tapoff[kGPairs];
#pragma unroll
    for (int j = 0; j < kGPairs; ++j) {
        const int t0 = pair_tap(STRIDE, j, 0), t1 = pair_tap(STRIDE, j, 1) >= 0 ? pair_tap(STRIDE, j, 1) : t0;
        const int cls = pair_class(STRIDE, j);
        const int sh0 = (tap_shift(STRIDE, cls >> 1, t0 / 3) * G::kHaloCols + tap_shift(STRIDE, cls & 1, t0 % 3)) * kGPitch;
        const int sh1 = (tap_shift(STRIDE, cls >> 1, t1 / 3) * G::kHaloCols + tap_shift(STRIDE, cls & 1, t1 % 3)) * kGPitch;
        tapoff[j] = (uint32_t)(((oct >> 1) ? sh1 : sh0) + px * kGPitch + (oct & 1) * 16);
    }
    // result register r of lane (px, oct): channel 4 oct + r of the input pixel of grid position (row, 16 cg + px)
#pragma unroll
    for (int row = 0; row < 2; ++row)
#pragma unroll
        for (int cg = 0; cg < 2; ++cg)
#pragma unroll
            for (int cls = 0; cls < G::kClasses; ++cls) {
                const int h = STRIDE * (i0 + 2 * wave + row) + (cls >> 1), w = STRIDE * (j0 + 16 * cg + px) + (cls & 1);
                const bool live = h < p.H && w < p.Wd;
                uint16_t* dst = p.dD + ((size_t)(b * p.H + h) * p.Wd + w) * p.C + oct * 4;
#pragma unroll
                for (int g = 0; g < kGSlab; ++g) {
                    f32x4g a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < kGPairs; ++j) {
                        if (pair_class(STRIDE, j) != cls) continue;
                        const uint32_t off = tapoff[j] + (uint32_t)(((2 * wave + row) * G::kHaloCols + 16 * cg) * kGPitch + g * 32);
                        const bf16x8_t gf = __builtin_bit_cast(bf16x8_t, *(SDGP_LDSG u32x4_t*)(smem + off));
                        a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[g][j], gf, a, 0, 0, 0);
                    }
                    if (live && g0 + g < p.groups) {
                        typedef uint32_t u32x2g __attribute__((ext_vector_type(2)));
                        const u32x2g v = {float2_to_bf16x2(a[0], a[1]), float2_to_bf16x2(a[2], a[3])};
                        *reinterpret_cast<u32x2g*>(dst + (g0 + g) * kGW) = v;
                    }
                }
            }
}

template <int STRIDE, int M, int RK, bool PRUNE, bool NLE2>
int launch_group16(const GroupedParams& p, hipStream_t stream) {
    auto kern = bwd_group16<STRIDE, M, RK, PRUNE, NLE2>;
    constexpr int lds = GroupedGeom<STRIDE>::kLds;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)((int64_t)p.B * p.tiles_h * p.tiles_w * p.slabs)), dim3(256), lds, stream, p);
    return launch_status();
}

template <int STRIDE, int M, bool NLE2>
int launch_group16_rk(const GroupedParams& p, int rk, hipStream_t stream) {
    if (rk == kRandom) return launch_group16<STRIDE, M, kRandom, true, NLE2>(p, stream);
    if (rk == kGreedy) return launch_group16<STRIDE, M, kGreedy, true, NLE2>(p, stream);
    return launch_group16<STRIDE, M, kAdjusted, true, NLE2>(p, stream);
}

template <int STRIDE>
int launch_group16_nm(const GroupedParams& p, int n, int m, int rk, hipStream_t stream) {
    if (n == m) return launch_group16<STRIDE, 4, kGreedy, false, true>(p, stream);
    const bool le2 = n <= 2;
    if (m == 4) return le2 ? launch_group16_rk<STRIDE, 4, true>(p, rk, stream) : launch_group16_rk<STRIDE, 4, false>(p, rk, stream);
    if (m == 8) return le2 ? launch_group16_rk<STRIDE, 8, true>(p, rk, stream) : launch_group16_rk<STRIDE, 8, false>(p, rk, stream);
    return le2 ? launch_group16_rk<STRIDE, 16, true>(p, rk, stream) : launch_group16_rk<STRIDE, 16, false>(p, rk, stream);
}

bool group16_fits(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int64_t groups,
                  int dt, int n, int m) {
    if (dt != SDGP_BF16 || groups < 1 || C_in != groups * kGW || C_out != groups * kGW) return false;
    if (R != 3 || S != 3 || (stride != 1 && stride != 2) || pad != 1 || B < 1 || H < 1 || Wd < 1) return false;
    if (n != m && !(m == 4 || m == 8 || m == 16)) return false;
    const int64_t gh = (H + stride - 1) / stride, gw = (Wd + stride - 1) / stride;   // the grid the tiles cover
    const int64_t tiles = B * ((gh + kGTH - 1) / kGTH) * ((gw + kGTW - 1) / kGTW) * ((groups + kGSlab - 1) / kGSlab);
    return tiles < INT32_MAX && H * Wd * C_out < ((int64_t)1 << 30) && B * H * Wd < INT32_MAX;
}

}  // namespace

// Workspace bytes of the matrix-core kernel for grouped layers (the re-indexed filter), or 0 when it does not take the
// problem.
size_t bwd_grouped_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad,
                             int64_t groups, int dt, int n, int m) {
    return group16_fits(B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt, n, m) ? (size_t)groups * kGImageBytes : 0;
}

// SDGP_OK after launching, a positive value when the problem does not fit (or the pointers are not 16-byte aligned),
// or a negative sdgp_status.  workspace: bwd_grouped_workspace(...) bytes.
int bwd_grouped_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R,
                       int S, int stride, int pad, int64_t groups, int dt, int n, int m, int rk, uint64_t seed, void* workspace,
                       hipStream_t stream) {
    if (!group16_fits(B, H, Wd, C_in, C_out, R, S, stride, pad, groups, dt, n, m)) return 1;
    if (workspace == nullptr || !is_aligned16(workspace) || !is_aligned16(dO) || (reinterpret_cast<uintptr_t>(dD) & 7u) != 0) return 1;
    GroupedParams p{};
    p.dO = static_cast<const uint16_t*>(dO), p.wimg = static_cast<const unsigned char*>(workspace), p.dD = static_cast<uint16_t*>(dD);
    p.B = (int)B, p.H = (int)H, p.Wd = (int)Wd, p.C = (int)C_out, p.groups = (int)groups;
    p.P = (int)((H + 2 - 3) / stride + 1), p.Q = (int)((Wd + 2 - 3) / stride + 1);
    const int64_t gh = (H + stride - 1) / stride, gw = (Wd + stride - 1) / stride;
    p.tiles_h = (int)((gh + kGTH - 1) / kGTH), p.tiles_w = (int)((gw + kGTW - 1) / kGTW), p.slabs = (int)((groups + kGSlab - 1) / kGSlab);
    p.n = n, p.mix = seed_mix(seed);
    hipLaunchKernelGGL(grouped_w_image, dim3((unsigned)(groups * kGPairs)), dim3(256), 0, stream, static_cast<const uint16_t*>(W),
                       static_cast<uint16_t*>(workspace), stride);
    return stride == 1 ? launch_group16_nm<1>(p, n, m, rk, stream) : launch_group16_nm<2>(p, n, m, rk, stream);
}

}  // namespace sdgp
