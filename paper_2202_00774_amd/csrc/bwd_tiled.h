// Tiled backward-data kernel on the gfx950 matrix cores (bf16 storage, fp32 accumulation).
//
// dL/dD = prune(dL/dO) (*) W as an implicit GEMM (Fig. 3 left; Sec. II-A maps the
// convolution to a matrix product): rows = input pixels, columns = input
// channels, reduction = taps x output channels -- the pruned axis (Fig. 1).
//
// Work decomposition
//   * A stride-s problem splits into s*s parity classes of input pixels; inside
//     a class the product is a stride-1 correlation with the sub-filter of taps
//     whose row/column offsets have that parity.  Each class has its own tap
//     list (dp, dq, weight offset); a class without taps is all zeros.
//   * A workgroup (4 wavefronts) owns a tile of TB images x TH x TW pixels of a
//     class (at most 256 rows) and BN columns.  Per chunk of KC reduction
//     channels it brings the halo of gradient pixels the taps reach into LDS
//     ONCE -- pruning each m-group on the way with the register ranker
//     (Sec. III-B), so a gradient element is ranked once per tile, not once per
//     tap -- and then walks the taps, streaming the matching W slab through a
//     double-buffered LDS stage.
//   * MODE 2 (n <= 2, m in {4,8,16}): the pruned halo is stored COMPRESSED, two
//     values and two 2-bit positions per aligned quad of channels, which is
//     what the structured-sparse matrix instruction v_smfmac_f32_32x32x32_bf16
//     consumes (every n<=2 pattern has at most two survivors per quad).  The
//     instruction reads 32 reduction channels per issue at the cost of 16.
//   * MODE 1 (other n:m): the pruned halo is stored dense with zeros and the
//     dense v_mfma_f32_32x32x16_bf16 is used; MODE 0 (n == m) skips the ranker.
//
// Operand layouts of the matrix instructions (measured on the device):
//   mfma 32x32x16:    A lane l holds row l%32, k = 8*(l/32)+e, e<8;  B lane l holds column l%32, same k;
//                     D lane l, register r holds column l%32, row 8*(r/4) + 4*(l/32) + r%4.
//   smfmac 32x32x32:  A lane l holds row l%32 and 8 compressed values covering dense k = 16*(l/32) .. +15,
//                     value e belongs to quad e/2 and sits at position (idx >> 2e) & 3 of it;
//                     B lane l holds column l%32, element eb: k = 16*(eb/8) + 8*(l/32) + eb%8;  D as above.
//   ds_read_b64_tr_b16: inside 16 lanes, lane i receives element i%4 of lanes i/4, 4+i/4, 8+i/4, 12+i/4.
//                     With lane L addressing row L/4, columns 4*(L%4).. of a row-major [k][n] slab, lane i
//                     ends up with column i for four consecutive k: a B fragment straight from the
//                     layout W has in memory (channels-in contiguous), no transposing store needed.
#pragma once

#include "ranker.h"

namespace sdgp {

constexpr int kMaxTaps = 49;
constexpr int kMaxClasses = 4;
constexpr int kTileRows = 256;

struct TapEntry {
    int dp, dq;  // gradient pixel = class pixel + (dp, dq)
    int woff;    // element offset of W[., r, s, 0] inside a W row: (r*S + s) * C_in
};

struct TileClass {
    int ph, pw;                      // parity of the input pixels of this class
    int HH, WW;                      // class grid: h = ph + stride*hh, hh < HH
    int tiles_h, tiles_w;            // tiles per image
    int tile_base;                   // first row-tile index of the class
    int tap_begin, tap_count;        // slice of taps[]
    int dpmin, dqmin;                // halo origin relative to the tile origin
    int HTH, HTW;                    // halo size = tile + tap range
};

struct TiledParams {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    int B, P, Q, C_out, C_in, H, Wd, stride;
    int w_row;                       // elements per W row: R*S*C_in
    int n;
    uint32_t mix;
    int TB, TH, TW;                  // tile shape in the class grid
    int ntiles_n, nblocks;
    int nclass;
    int halo_max;                    // largest TB*HTH*HTW over classes
    TileClass cls[kMaxClasses];
    TapEntry taps[kMaxTaps];
};

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16_t __attribute__((ext_vector_type(16)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

#define SDGP_LDS __attribute__((address_space(3)))

template <int BN, int KC, int MODE>
struct TiledLayout {
    static constexpr bool kSparse = MODE == 2;
    static constexpr int kAPixBytes = kSparse ? KC : KC * 2;
    static constexpr int kAPitch = kAPixBytes + 16;
    static constexpr int kMetaPitch = KC / 8;
    static constexpr int kWPitch = BN * 2 + 32;
    static constexpr int kWStage = KC * kWPitch;
    // byte offsets inside dynamic LDS
    __host__ __device__ static int off_w() { return 0; }
    __host__ __device__ static int off_rowpix() { return 2 * kWStage; }
    __host__ __device__ static int off_halopix() { return off_rowpix() + kTileRows * 4; }
    __host__ __device__ static int off_a(int halo) { return (off_halopix() + halo * 4 + 15) & ~15; }
    __host__ __device__ static int off_meta(int halo) { return off_a(halo) + halo * kAPitch; }
    __host__ __device__ static int total(int halo) { return off_meta(halo) + (kSparse ? halo * kMetaPitch : 0); }
};

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

template <int BN, int KC, int MODE, int M, int RK>
__global__ void __launch_bounds__(256, 2) bwd_tiled(const TiledParams p) {
    using L = TiledLayout<BN, KC, MODE>;
    constexpr bool SPARSE = MODE == 2;
    constexpr int WAVES_N = BN / 64;
    constexpr int WAVES_M = 4 / WAVES_N;
    constexpr int WM = kTileRows / WAVES_M;
    constexpr int TM = WM / 32;  // 32-row tiles per wave
    constexpr int TN = 2;        // 32-column tiles per wave (64 columns)
    constexpr int ITEM = (MODE == 1 && M > 16) ? M : 16;  // channels a lane prunes at a time
    constexpr int ITEMS_PER_PIX = KC / ITEM;
    constexpr int KSTEP = SPARSE ? 32 : 16;

    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDS unsigned char* smem = (SDGP_LDS unsigned char*)smem_generic;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- which tile: consecutive logical ids stay on one XCD (hardware deals workgroups round-robin over 8 XCDs)
    int lid = blockIdx.x;
    {
        const int per = p.nblocks >> 3;
        if (lid < (per << 3)) lid = (lid & 7) * per + (lid >> 3);
    }
    const int ntile = lid % p.ntiles_n;
    const int mtile = lid / p.ntiles_n;
    int ci = 0;
#pragma unroll
    for (int c = 1; c < kMaxClasses; ++c)
        if (c < p.nclass && mtile >= p.cls[c].tile_base) ci = c;
    const TileClass cl = p.cls[ci];
    const int tt = mtile - cl.tile_base;
    const int tw_i = tt % cl.tiles_w;
    const int th_i = (tt / cl.tiles_w) % cl.tiles_h;
    const int tb_i = tt / (cl.tiles_w * cl.tiles_h);
    const int b0 = tb_i * p.TB, hh0 = th_i * p.TH, ww0 = tw_i * p.TW;
    const int n0 = ntile * BN;
    const int tile_rows = p.TB * p.TH * p.TW;
    const int tile_hw = p.TH * p.TW;
    const int halo_hw = cl.HTH * cl.HTW;
    const int nhalo = p.TB * halo_hw;

    SDGP_LDS int* rowpix = (SDGP_LDS int*)(smem + L::off_rowpix());
    SDGP_LDS int* halopix = (SDGP_LDS int*)(smem + L::off_halopix());
    SDGP_LDS unsigned char* lds_w = smem + L::off_w();
    SDGP_LDS unsigned char* lds_a = smem + L::off_a(p.halo_max);
    SDGP_LDS unsigned char* lds_meta = smem + L::off_meta(p.halo_max);

    // ---- tables: output pixel of every tile row, gradient pixel of every halo position (-1 = none)
    {
        const int m = tid;
        int pix = -1;
        if (m < tile_rows) {
            const int tb = m / tile_hw, rem = m % tile_hw;
            const int th = rem / p.TW, tw = rem % p.TW;
            const int b = b0 + tb, hh = hh0 + th, ww = ww0 + tw;
            if (b < p.B && hh < cl.HH && ww < cl.WW)
                pix = (b * p.H + cl.ph + p.stride * hh) * p.Wd + cl.pw + p.stride * ww;
        }
        rowpix[m] = pix;
        for (int hp = tid; hp < nhalo; hp += 256) {
            const int tb = hp / halo_hw, rem = hp % halo_hw;
            const int hy = rem / cl.HTW, hx = rem % cl.HTW;
            const int b = b0 + tb, pp = hh0 + hy + cl.dpmin, qq = ww0 + hx + cl.dqmin;
            const bool ok = b < p.B && pp >= 0 && pp < p.P && qq >= 0 && qq < p.Q;
            halopix[hp] = ok ? (b * p.P + pp) * p.Q + qq : -1;
        }
    }

    // ---- per-lane fragment addresses
    int a_lane[TM], meta_lane[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        const int m = wm * WM + t * 32 + (lane & 31);
        int base = 0;
        if (m < tile_rows) {
            const int tb = m / tile_hw, rem = m % tile_hw;
            base = (tb * cl.HTH + rem / p.TW) * cl.HTW + rem % p.TW;
        }
        a_lane[t] = base * L::kAPitch + (lane >> 5) * 16;
        meta_lane[t] = base * L::kMetaPitch + (lane >> 5) * 2;
    }
    const int b_lane = (8 * (lane >> 5) + ((lane & 15) >> 2)) * L::kWPitch + (wn * 64 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int u = 0; u < TN; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.0f;

    // W slab loader: KC rows x BN columns, 16-byte vectors.
    constexpr int W_VECS = KC * BN / 8 / 256;  // per thread
    u32x4_t wreg[W_VECS];
    auto load_w = [&](int kc0, const TapEntry& tp) {
#pragma unroll
        for (int i = 0; i < W_VECS; ++i) {
            const int v = tid + i * 256;
            const int row = v / (BN / 8), cv = v % (BN / 8);
            const int k = kc0 + row, c = n0 + cv * 8;
            u32x4_t x = {0u, 0u, 0u, 0u};
            if (k < p.C_out && c < p.C_in)
                x = *reinterpret_cast<const u32x4_t*>(p.W + (size_t)k * p.w_row + tp.woff + c);
            wreg[i] = x;
        }
    };
    auto store_w = [&](int buf) {
#pragma unroll
        for (int i = 0; i < W_VECS; ++i) {
            const int v = tid + i * 256;
            const int row = v / (BN / 8), cv = v % (BN / 8);
            *(SDGP_LDS u32x4_t*)(lds_w + buf * L::kWStage + row * L::kWPitch + cv * 16) = wreg[i];
        }
    };

    for (int kc0 = 0; kc0 < p.C_out && cl.tap_count > 0; kc0 += KC) {
        __syncthreads();  // tables written (first pass) / previous chunk fully consumed

        // ---- halo of this channel chunk -> LDS, pruned on the way
        for (int it = tid; it < nhalo * ITEMS_PER_PIX; it += 256) {
            const int hp = it / ITEMS_PER_PIX, part = it % ITEMS_PER_PIX;
            const int gp = halopix[hp];
            const int k = kc0 + part * ITEM;
            constexpr int NV = ITEM / 8;
            u32x4_t v[NV];
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                v[i] = u32x4_t{0u, 0u, 0u, 0u};
                if (gp >= 0 && k + i * 8 < p.C_out)
                    v[i] = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4_t*>(p.dO + (size_t)gp * p.C_out + k + i * 8));
            }
            if constexpr (MODE == 0) {
#pragma unroll
                for (int i = 0; i < NV; ++i)
                    *(SDGP_LDS u32x4_t*)(lds_a + hp * L::kAPitch + part * (ITEM * 2) + i * 16) = v[i];
            } else {
                uint32_t raw[ITEM], out[ITEM];
                bool keep[ITEM];
#pragma unroll
                for (int i = 0; i < NV; ++i)
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        raw[i * 8 + 2 * w] = v[i][w] & 0xFFFFu;
                        raw[i * 8 + 2 * w + 1] = v[i][w] >> 16;
                    }
                const uint64_t e0 = (uint64_t)(gp < 0 ? 0 : gp) * (uint64_t)p.C_out + (uint64_t)k;
#pragma unroll
                for (int g = 0; g < ITEM / M; ++g) {
                    uint32_t r[M], o[M];
                    bool kk[M];
#pragma unroll
                    for (int j = 0; j < M; ++j) r[j] = raw[g * M + j];
                    const uint64_t eg = e0 + (uint64_t)(g * M);  // a group never straddles a 2^32 boundary
                    prune_group<kBF16, M, RK, SPARSE>(r, p.n, hash_row(p.mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
                    for (int j = 0; j < M; ++j) {
                        out[g * M + j] = o[j];
                        keep[g * M + j] = kk[j];
                    }
                }
                if constexpr (MODE == 1) {
#pragma unroll
                    for (int i = 0; i < NV; ++i) {
                        u32x4_t x;
#pragma unroll
                        for (int w = 0; w < 4; ++w) x[w] = out[i * 8 + 2 * w] | (out[i * 8 + 2 * w + 1] << 16);
                        *(SDGP_LDS u32x4_t*)(lds_a + hp * L::kAPitch + part * (ITEM * 2) + i * 16) = x;
                    }
                } else {
                    uint32_t cv[8], meta = 0;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const bool kq[4] = {keep[4 * q], keep[4 * q + 1], keep[4 * q + 2], keep[4 * q + 3]};
                        const uint32_t oq[4] = {out[4 * q], out[4 * q + 1], out[4 * q + 2], out[4 * q + 3]};
                        uint32_t pos;
                        compress_quad(kq, oq, cv[2 * q], cv[2 * q + 1], pos);
                        meta |= pos << (4 * q);
                    }
                    const u32x4_t x = {cv[0] | (cv[1] << 16), cv[2] | (cv[3] << 16), cv[4] | (cv[5] << 16),
                                       cv[6] | (cv[7] << 16)};
                    *(SDGP_LDS u32x4_t*)(lds_a + hp * L::kAPitch + part * 16) = x;
                    *(SDGP_LDS uint16_t*)(lds_meta + hp * L::kMetaPitch + part * 2) = (uint16_t)meta;
                }
            }
        }

        load_w(kc0, p.taps[cl.tap_begin]);
        store_w(0);
        __syncthreads();

        for (int ti = 0; ti < cl.tap_count; ++ti) {
            const TapEntry tp = p.taps[cl.tap_begin + ti];
            const bool more = ti + 1 < cl.tap_count;
            if (more) load_w(kc0, p.taps[cl.tap_begin + ti + 1]);

            const int tap_off = (tp.dp - cl.dpmin) * cl.HTW + (tp.dq - cl.dqmin);
            SDGP_LDS unsigned char* wbuf = lds_w + (ti & 1) * L::kWStage + b_lane;
            SDGP_LDS unsigned char* abuf = lds_a + tap_off * L::kAPitch;
            SDGP_LDS unsigned char* mbuf = lds_meta + tap_off * L::kMetaPitch;
#pragma unroll
            for (int ks = 0; ks < KC / KSTEP; ++ks) {
                if constexpr (SPARSE) {
                    bf16x16_t bfrag[TN];
#pragma unroll
                    for (int u = 0; u < TN; ++u) {
                        s16x4_t q[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (SDGP_LDS s16x4_t*)(wbuf + (ks * 32 + (i >> 1) * 16 + (i & 1) * 4) * L::kWPitch + u * 64));
                        typedef short s16x16_t __attribute__((ext_vector_type(16)));
                        const s16x16_t all = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3],
                                              q[2][0], q[2][1], q[2][2], q[2][3], q[3][0], q[3][1], q[3][2], q[3][3]};
                        bfrag[u] = __builtin_bit_cast(bf16x16_t, all);
                    }
#pragma unroll
                    for (int t = 0; t < TM; ++t) {
                        const u32x4_t araw = *(SDGP_LDS u32x4_t*)(abuf + a_lane[t] + ks * 32);
                        const int meta = *(SDGP_LDS uint16_t*)(mbuf + meta_lane[t] + ks * 4);
                        const bf16x8_t afrag = __builtin_bit_cast(bf16x8_t, araw);
#pragma unroll
                        for (int u = 0; u < TN; ++u)
                            acc[t][u] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(afrag, bfrag[u], acc[t][u], meta, 0, 0);
                    }
                } else {
                    bf16x8_t bfrag[TN];
#pragma unroll
                    for (int u = 0; u < TN; ++u) {
                        s16x4_t q[2];
#pragma unroll
                        for (int i = 0; i < 2; ++i)
                            q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (SDGP_LDS s16x4_t*)(wbuf + (ks * 16 + i * 4) * L::kWPitch + u * 64));
                        typedef short s16x8_t __attribute__((ext_vector_type(8)));
                        const s16x8_t all = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3]};
                        bfrag[u] = __builtin_bit_cast(bf16x8_t, all);
                    }
#pragma unroll
                    for (int t = 0; t < TM; ++t) {
                        const u32x4_t araw = *(SDGP_LDS u32x4_t*)(abuf + a_lane[t] + ks * 32);
                        const bf16x8_t afrag = __builtin_bit_cast(bf16x8_t, araw);
#pragma unroll
                        for (int u = 0; u < TN; ++u)
                            acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[u], acc[t][u], 0, 0, 0);
                    }
                }
            }

            if (more) store_w((ti + 1) & 1);
            __syncthreads();
        }
    }
    if (cl.tap_count == 0) __syncthreads();  // rowpix must be visible

    // ---- epilogue: fp32 -> bf16 (RNE), NHWC store
#pragma unroll
    for (int t = 0; t < TM; ++t) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = wm * WM + t * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const int pix = rowpix[m];
            if (pix < 0) continue;
#pragma unroll
            for (int u = 0; u < TN; ++u) {
                const int c = n0 + wn * 64 + u * 32 + (lane & 31);
                if (c < p.C_in) p.dD[(size_t)pix * p.C_in + c] = (uint16_t)float_to_bf16(acc[t][u][r]);
            }
        }
    }
}

}  // namespace sdgp
