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
//     ring of LDS stages.
//   * The workgroup is split by role.  Wavefronts 0-3 (consumers) only read
//     fragments from LDS and issue matrix instructions; wavefronts 4-7
//     (producers) load W slabs and the next chunk's halo from global memory,
//     rank/prune/compress it and write LDS.  Each SIMD hosts one wave of each
//     role, so the ranker's integer work and the memory latency overlap the
//     matrix pipe instead of stalling it.  One barrier per (chunk, tap) stage
//     hands a W slot and, at chunk boundaries, a halo buffer from one role to
//     the other.
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

#include <type_traits>

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
    static constexpr int kWSlots = 3;
    // byte offsets inside dynamic LDS
    __host__ __device__ static int off_w() { return 0; }
    __host__ __device__ static int off_rowpix() { return kWSlots * kWStage; }
    __host__ __device__ static int off_halopix() { return off_rowpix() + kTileRows * 4; }
    __host__ __device__ static int off_a(int halo) { return (off_halopix() + halo * 4 + 15) & ~15; }
    __host__ __device__ static int a_bytes(int halo) { return halo * kAPitch; }
    __host__ __device__ static int meta_bytes(int halo) { return kSparse ? ((halo * kMetaPitch + 15) & ~15) : 0; }
    __host__ __device__ static int off_meta(int halo) { return off_a(halo) + 2 * a_bytes(halo); }
    __host__ __device__ static int total(int halo) { return off_meta(halo) + 2 * meta_bytes(halo); }
};

constexpr int kMaxHaloItems = 8;  // halo items (16 channels of one pixel) a producer lane holds in flight

// One halo item (ITEM channels of one gradient pixel, already in registers) -> LDS:
// verbatim (MODE 0), pruned with zeros (MODE 1) or pruned and compressed (MODE 2).
template <int KC, int MODE, int M, int RK, int ITEM>
__device__ __forceinline__ void halo_item_to_lds(const u32x4_t (&v)[ITEM / 8], int hp, int part, uint64_t e0, int n,
                                                 uint32_t mix, SDGP_LDS unsigned char* lds_a,
                                                 SDGP_LDS unsigned char* lds_meta) {
    constexpr bool SPARSE = MODE == 2;
    constexpr int NV = ITEM / 8;
    constexpr int APITCH = (SPARSE ? KC : KC * 2) + 16;
    if constexpr (MODE == 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) *(SDGP_LDS u32x4_t*)(lds_a + hp * APITCH + part * (ITEM * 2) + i * 16) = v[i];
    } else if constexpr (SPARSE) {
        static_assert(ITEM == 16, "the compressing rankers take sixteen channels");
        const uint32_t w[8] = {v[0][0], v[0][1], v[0][2], v[0][3], v[1][0], v[1][1], v[1][2], v[1][3]};
        uint32_t packed[4], meta;
        prune_compress16<M, RK>(w, n, mix, e0, packed, meta);
        const u32x4_t x = {packed[0], packed[1], packed[2], packed[3]};
        *(SDGP_LDS u32x4_t*)(lds_a + hp * APITCH + part * 16) = x;
        *(SDGP_LDS uint16_t*)(lds_meta + hp * (KC / 8) + part * 2) = (uint16_t)meta;
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
#pragma unroll
        for (int g = 0; g < ITEM / M; ++g) {
            uint32_t r[M], o[M];
            bool kk[M];
#pragma unroll
            for (int j = 0; j < M; ++j) r[j] = raw[g * M + j];
            const uint64_t eg = e0 + (uint64_t)(g * M);  // a group never straddles a 2^32 boundary
            prune_group<kBF16, M, RK, false>(r, n, hash_row(mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
            for (int j = 0; j < M; ++j) {
                out[g * M + j] = o[j];
                keep[g * M + j] = kk[j];
            }
        }
        // MODE 1: the pruned channels stay in place, zeros where dropped
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            u32x4_t x;
#pragma unroll
            for (int w = 0; w < 4; ++w) x[w] = out[i * 8 + 2 * w] | (out[i * 8 + 2 * w + 1] << 16);
            *(SDGP_LDS u32x4_t*)(lds_a + hp * APITCH + part * (ITEM * 2) + i * 16) = x;
        }
    }
}

template <int BN, int KC, int MODE, int M, int RK>
__global__ void __launch_bounds__(512) bwd_tiled(const TiledParams p) {
    using L = TiledLayout<BN, KC, MODE>;
    constexpr bool SPARSE = MODE == 2;
    constexpr int WAVES_N = BN / 64;
    constexpr int WAVES_M = 4 / WAVES_N;
    constexpr int WM = kTileRows / WAVES_M;
    constexpr int TM = WM / 32;  // 32-row tiles per consumer wave
    constexpr int TN = 2;        // 32-column tiles per consumer wave (64 columns)
    constexpr int ITEM = (MODE == 1 && M > 16) ? M : 16;  // channels a lane prunes at a time
    constexpr int ITEMS_PER_PIX = KC / ITEM;
    constexpr int NV = ITEM / 8;
    constexpr int KSTEP = SPARSE ? 32 : 16;
    constexpr int NKS = KC / KSTEP;
    constexpr int W_VECS = KC * BN / 8 / 256;  // 16-byte vectors of a W slab per producer lane

    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDS unsigned char* smem = (SDGP_LDS unsigned char*)smem_generic;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool producer = wave >= 4;
    const int cw = wave & 3;  // index inside the role
    const int wm = cw / WAVES_N, wn = cw % WAVES_N;
    const int ptid = tid & 255;

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
    const int ntaps = cl.tap_count;
    const int nchunks = (p.C_out + KC - 1) / KC;
    const int nstages = ntaps * nchunks;

    SDGP_LDS int* rowpix = (SDGP_LDS int*)(smem + L::off_rowpix());
    SDGP_LDS int* halopix = (SDGP_LDS int*)(smem + L::off_halopix());
    SDGP_LDS unsigned char* lds_w = smem + L::off_w();
    SDGP_LDS unsigned char* lds_a = smem + L::off_a(p.halo_max);
    SDGP_LDS unsigned char* lds_meta = smem + L::off_meta(p.halo_max);
    const int a_buf_bytes = L::a_bytes(p.halo_max), meta_buf_bytes = L::meta_bytes(p.halo_max);

    // ---- tables: output pixel of every tile row, gradient pixel of every halo position (-1 = none)
    if (tid < kTileRows) {
        const int m = tid;
        int pix = -1;
        if (m < tile_rows) {
            const int tb = m / tile_hw, rem = m % tile_hw;
            const int th = rem / p.TW, tw = rem % p.TW;
            const int b = b0 + tb, hh = hh0 + th, ww = ww0 + tw;
            if (b < p.B && hh < cl.HH && ww < cl.WW) pix = (b * p.H + cl.ph + p.stride * hh) * p.Wd + cl.pw + p.stride * ww;
        }
        rowpix[m] = pix;
    }
    for (int hp = tid; hp < nhalo; hp += 512) {
        const int tb = hp / halo_hw, rem = hp % halo_hw;
        const int hy = rem / cl.HTW, hx = rem % cl.HTW;
        const int b = b0 + tb, pp = hh0 + hy + cl.dpmin, qq = ww0 + hx + cl.dqmin;
        const bool ok = b < p.B && pp >= 0 && pp < p.P && qq >= 0 && qq < p.Q;
        halopix[hp] = ok ? (b * p.P + pp) * p.Q + qq : -1;
    }
    __syncthreads();

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int u = 0; u < TN; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.0f;

    if (nstages > 0) {
        if (producer) {
            // =========================================================== producers
            const int nitems = nhalo * ITEMS_PER_PIX;
            const int my_items = (nitems - ptid + 255) / 256;  // items ptid, ptid+256, ... (at most kMaxHaloItems)

            auto load_w = [&](u32x4_t (&w)[W_VECS], int chunk, int ti) {
                const int woff = p.taps[cl.tap_begin + ti].woff;
#pragma unroll
                for (int i = 0; i < W_VECS; ++i) {
                    const int v = ptid + i * 256;
                    const int row = v / (BN / 8), cv = v % (BN / 8);
                    const int k = chunk * KC + row, c = n0 + cv * 8;
                    u32x4_t x = {0u, 0u, 0u, 0u};
                    if (k < p.C_out && c < p.C_in) x = *reinterpret_cast<const u32x4_t*>(p.W + (size_t)k * p.w_row + woff + c);
                    w[i] = x;
                }
            };
            auto store_w = [&](const u32x4_t (&w)[W_VECS], int slot) {
#pragma unroll
                for (int i = 0; i < W_VECS; ++i) {
                    const int v = ptid + i * 256;
                    const int row = v / (BN / 8), cv = v % (BN / 8);
                    *(SDGP_LDS u32x4_t*)(lds_w + slot * L::kWStage + row * L::kWPitch + cv * 16) = w[i];
                }
            };
            auto load_item = [&](u32x4_t (&v)[NV], int j, int chunk) {
                const int it = ptid + j * 256;
                const int hp = it / ITEMS_PER_PIX, part = it % ITEMS_PER_PIX;
                const int gp = (it < nitems) ? halopix[hp] : -1;
                const int k = chunk * KC + part * ITEM;
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                    v[i] = u32x4_t{0u, 0u, 0u, 0u};
                    if (gp >= 0 && k + i * 8 < p.C_out)
                        v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p.dO + (size_t)gp * p.C_out + k + i * 8));
                }
            };
            auto finish_item = [&](const u32x4_t (&v)[NV], int j, int chunk) {
                const int it = ptid + j * 256;
                if (it >= nitems) return;
                const int hp = it / ITEMS_PER_PIX, part = it % ITEMS_PER_PIX;
                const int gp = halopix[hp];
                const uint64_t e0 = (uint64_t)(gp < 0 ? 0 : gp) * (uint64_t)p.C_out + (uint64_t)(chunk * KC + part * ITEM);
                halo_item_to_lds<KC, MODE, M, RK, ITEM>(v, hp, part, e0, p.n, p.mix, lds_a + (chunk & 1) * a_buf_bytes,
                                                        lds_meta + (chunk & 1) * meta_buf_bytes);
            };

            u32x4_t hreg[kMaxHaloItems][NV];
            u32x4_t wA[W_VECS], wB[W_VECS];

            // prologue: halo of chunk 0, W stages 0 and 1 in LDS; stages 2 and 3 in flight
#pragma unroll
            for (int j = 0; j < kMaxHaloItems; ++j)
                if (j < my_items) load_item(hreg[j], j, 0);
            load_w(wA, 0, 0);
            if (nstages > 1) load_w(wB, 1 / ntaps, 1 % ntaps);
            store_w(wA, 0);
            if (nstages > 1) store_w(wB, 1);
#pragma unroll
            for (int j = 0; j < kMaxHaloItems; ++j)
                if (j < my_items) finish_item(hreg[j], j, 0);
            if (nstages > 2) load_w(wA, 2 / ntaps, 2 % ntaps);
            if (nstages > 3) load_w(wB, 3 / ntaps, 3 % ntaps);
            __syncthreads();

            // Stage s is consumed during step s.  In step s the producers write stage s+2 (loaded two steps ago)
            // into its ring slot and issue the loads of stage s+4.  The halo of chunk c+1 is requested in the
            // first step of chunk c and ranked/pruned/written in the later steps of that chunk.
            int chunk = 0, ti = 0;           // (chunk, tap) of stage s
            int c2 = 2 / ntaps, t2 = 2 % ntaps;  // of stage s+2 ... advanced incrementally
            int c4 = 4 / ntaps, t4 = 4 % ntaps;  // of stage s+4
            const int spread = ntaps >= 3 ? ntaps - 2 : 1;  // steps 1 .. spread finish the next halo (a step early when possible)
            auto step = [&](int s, u32x4_t (&w)[W_VECS]) {
                if (s + 2 < nstages) store_w(w, (s + 2) % L::kWSlots);
                if (s + 4 < nstages) load_w(w, c4, t4);
                if (chunk + 1 < nchunks) {
                    if (ntaps == 1) {
#pragma unroll
                        for (int j = 0; j < kMaxHaloItems; ++j)
                            if (j < my_items) load_item(hreg[j], j, chunk + 1);
#pragma unroll
                        for (int j = 0; j < kMaxHaloItems; ++j)
                            if (j < my_items) finish_item(hreg[j], j, chunk + 1);
                    } else if (ti == 0) {
#pragma unroll
                        for (int j = 0; j < kMaxHaloItems; ++j)
                            if (j < my_items) load_item(hreg[j], j, chunk + 1);
                    } else {
#pragma unroll
                        for (int j = 0; j < kMaxHaloItems; ++j)
                            if (j < my_items && (j % spread) == ti - 1) finish_item(hreg[j], j, chunk + 1);
                    }
                }
                if (++ti == ntaps) ti = 0, ++chunk;
                if (++t2 == ntaps) t2 = 0, ++c2;
                if (++t4 == ntaps) t4 = 0, ++c4;
                __syncthreads();
            };
            for (int s = 0; s < nstages; s += 2) {
                step(s, wA);
                if (s + 1 < nstages) step(s + 1, wB);
            }
        } else {
            // =========================================================== consumers
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
            const int b_lane = (8 * (lane >> 5) + ((lane & 15) >> 2)) * L::kWPitch +
                               (wn * 64 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
            __syncthreads();  // matches the producers' prologue barrier

            // tap -> halo offset, one tap per lane, fetched with readlane (no memory access in the loop)
            int my_tap_off = 0;
            if (lane < ntaps) {
                const TapEntry tp = p.taps[cl.tap_begin + lane];
                my_tap_off = (tp.dp - cl.dpmin) * cl.HTW + (tp.dq - cl.dqmin);
            }

            struct Frags {
                bf16x8_t a[TM];
                int meta[TM];
                typename std::conditional<SPARSE, bf16x16_t, bf16x8_t>::type b[TN];
            };
            // All fragments of one k-step of one stage.
            auto load_frags = [&](Frags& f, int slot, int chunk, int ti, int ks) {
                const int tap_off = __builtin_amdgcn_readlane(my_tap_off, ti);
                SDGP_LDS unsigned char* wbuf = lds_w + slot * L::kWStage + b_lane;
                SDGP_LDS unsigned char* abuf = lds_a + (chunk & 1) * a_buf_bytes + tap_off * L::kAPitch;
#pragma unroll
                for (int t = 0; t < TM; ++t) {
                    const u32x4_t araw = *(SDGP_LDS u32x4_t*)(abuf + a_lane[t] + ks * 32);
                    f.a[t] = __builtin_bit_cast(bf16x8_t, araw);
                }
                if constexpr (SPARSE) {
                    SDGP_LDS unsigned char* mbuf = lds_meta + (chunk & 1) * meta_buf_bytes + tap_off * L::kMetaPitch;
#pragma unroll
                    for (int t = 0; t < TM; ++t) f.meta[t] = *(SDGP_LDS uint16_t*)(mbuf + meta_lane[t] + ks * 4);
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
                        f.b[u] = __builtin_bit_cast(bf16x16_t, all);
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < TN; ++u) {
                        s16x4_t q[2];
#pragma unroll
                        for (int i = 0; i < 2; ++i)
                            q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (SDGP_LDS s16x4_t*)(wbuf + (ks * 16 + i * 4) * L::kWPitch + u * 64));
                        typedef short s16x8_t __attribute__((ext_vector_type(8)));
                        const s16x8_t all = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3]};
                        f.b[u] = __builtin_bit_cast(bf16x8_t, all);
                    }
                }
            };
            auto mma = [&](const Frags& f) {
#pragma unroll
                for (int t = 0; t < TM; ++t)
#pragma unroll
                    for (int u = 0; u < TN; ++u) {
                        if constexpr (SPARSE)
                            acc[t][u] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[t], f.b[u], acc[t][u], f.meta[t], 0, 0);
                        else
                            acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[t], f.b[u], acc[t][u], 0, 0, 0);
                    }
            };

            // The fragments of k-step q+1 are requested before the matrix instructions of k-step q issue.
            // The next stage's W slot is always ready one step ahead; its halo buffer is ready ahead only
            // inside a chunk, or across chunks when the producers finish the halo a step early (ntaps >= 3).
            static_assert(NKS % 2 == 0, "fragment double buffering alternates per k-step");
            const bool early_halo = ntaps >= 3;
            Frags fr[2];
            int chunk = 0, ti = 0, slot = 0;
            load_frags(fr[0], 0, 0, 0, 0);
            for (int s = 0; s < nstages; ++s) {
                int nti = ti + 1, nchunk = chunk, nslot = slot + 1;
                if (nti == ntaps) nti = 0, ++nchunk;
                if (nslot == L::kWSlots) nslot = 0;
                const bool has_next = s + 1 < nstages;
                const bool ahead = has_next && (nchunk == chunk || early_halo);
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    if (ks + 1 < NKS) load_frags(fr[(ks + 1) & 1], slot, chunk, ti, ks + 1);
                    else if (ahead) load_frags(fr[0], nslot, nchunk, nti, 0);
                    mma(fr[ks & 1]);
                }
                __syncthreads();
                if (has_next && !ahead) load_frags(fr[0], nslot, nchunk, nti, 0);
                ti = nti, chunk = nchunk, slot = nslot;
            }
        }
    }

    // ---- epilogue (consumers): fp32 -> bf16 (RNE), NHWC store
    if (!producer) {
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
}

}  // namespace sdgp
