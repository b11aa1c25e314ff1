// Backward-data kernel for stride-1 filters that are three taps wide (3x3, 2x3, 1x3): one filter ROW per stage.
// dL/dD = prune(dL/dO) (*) W as an implicit GEMM (Fig. 3 left; Sec. II-A): rows = input pixels, columns = input
// channels, reduction = taps x output channels, the pruned axis (Fig. 1).
//
// Design, from measurements on gfx950:
//   * Eight wavefronts, all of one kind: each owns a 128 x 64 register tile of a 512-row x 128-column workgroup tile
//     (smaller tiles: 256 rows when 512-row tiles cannot fill the chip, 64 columns when C_in <= 64) and issues its
//     share of the copies itself.  Two matrix wavefronts per SIMD keep the matrix pipe fed while the other one waits
//     for LDS; tiles of this size keep the LDS read traffic (about 96 KB per 1024 matrix cycles) below what the LDS
//     delivers.  Dedicated copy wavefronts would cost the registers that such tiles need.
//   * Every byte from global memory moves with direct-to-LDS loads (lane i of a wavefront writes 16 bytes at LDS
//     base + 16 i); they need no registers.
//   * The reduction runs in chunks of 32 channels.  One stage = (chunk, filter row): three taps, 48 dense or 24
//     sparse matrix instructions per wavefront between two barriers.  What a stage costs besides its matrix
//     instructions -- the barrier and the wait in front of it, the copies and their bookkeeping, the skew between
//     wavefronts -- is paid once per three taps.
//   * The gradient halo of a tile (the pixels its taps reach, clipped to the image) is brought in ONCE per chunk and
//     shared by all taps; a per-(tap, row) table in LDS maps a tile row to its halo pixel (a zero pixel for taps
//     outside the image), so nothing is stored or copied for the padding.
//   * The result leaves through LDS: fp32 -> bf16, then 16-byte stores of whole pixel rows.
//   * W: the three slabs of the next stage's filter row are requested at the start of a stage into the other half of
//     a two-set ring and are complete at the barrier that ends it (a stage lasts several copy latencies).
//   * Dense: the next chunk's halo is copied into the other halo buffer, a share per stage.
//   * Pruning (Sec. III-B): stage r of a chunk ranks / prunes / compresses share r of the next chunk's halo -- one
//     16-channel item per lane of the whole workgroup -- from a raw slot that the previous stage filled, and requests
//     the raw share of the stage after it.  Output: two values + two 2-bit positions per aligned quad of channels,
//     the operand of v_smfmac_f32_32x32x32_bf16.
//   * Nothing is read across a barrier except the address table, so every request counter can simply drain
//     (s_waitcnt vmcnt(0)) before the barrier: no copy has to be counted, no stand-in copies are needed.
#pragma once

#include <type_traits>

#include "lds_copy.h"

namespace sdgp {

struct RowParams {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    int B, P, Q, C_out, C_in, H, Wd;
    int R, pad;                  // R filter rows of three taps each
    int w_row;                   // elements per W row: R*3*C_in
    int n;
    uint32_t mix;
    int TB, TH, TW;              // tile: TB images x TH x TW pixels (<= the kernel's ROWS)
    int tiles_h, tiles_w;
    int halo_max;                // upper bound of the halo pixels of any tile (LDS sizing)
    int npad;                    // positions of the zero-padded halo grid of a tile: TB * (TH + R - 1) * (TW + 2)
    int ups;                     // halo copy units per stage: a 1/R share of the halo, at most 16
    int ntiles_n, nblocks;
};

constexpr int kRowKC = 32;         // reduction channels per chunk
constexpr int kRowTaps = 3;        // taps per stage (filter width)
constexpr int kRowMaxRows = 3;

template <int BN, int MODE, int ROWS>
struct RowLayout {
    static constexpr bool kSparse = MODE == 2;
    static constexpr bool kPrunes = MODE != 0;  // raw halo shares are staged and ranked (MODE 1 stores them dense, zero-filled)
    static constexpr int kWRow = BN * 2;
    static constexpr int kWSlab = kRowKC * kWRow;
    static constexpr int kWUnits = kWSlab / 1024;
    static constexpr int kWSet = kRowTaps * kWSlab;            // the slabs of one filter row
    static constexpr int kAPitch = 64;                         // dense and zero-filled halo: 32 channels per pixel
    static constexpr int kRawSlot = 16 * 1024;
    static constexpr int kOutPitch = BN * 2 + 16;
    __host__ __device__ static int pad16(int halo) { return (halo + 15) & ~15; }
    __host__ __device__ static int pixels(int halo) { return pad16(halo) + 16; }  // + one all-zero pixel
    __host__ __device__ static int zero_pixel(int halo) { return pad16(halo); }
    // Compressed halo (kSparse): a zero-padded grid of `npad` positions, in planes -- per buffer two planes of kept
    // values (16 bytes per position: the eight survivors of sixteen channels) and two planes of their 2-bit positions
    // (2 bytes per position), one plane per half of the 32-channel chunk.  Plane sizes are 128 modulo 256 bytes, so
    // the two planes a wavefront touches in one access fall into different halves of the banks.
    __host__ __device__ static int plane_a(int npad) { return ((npad * 16 + 255) & ~255) + 128; }
    __host__ __device__ static int plane_m(int npad) { return ((npad * 2 + 255) & ~255) + 128; }
    __host__ __device__ static int off_rowpix() { return 0; }
    __host__ __device__ static int off_out() { return ROWS * 4; }
    __host__ __device__ static int off_w() { return off_out(); }
    __host__ __device__ static int off_atab() { return off_w() + 2 * kWSet; }
    __host__ __device__ static int off_haloaddr() { return off_atab() + (kSparse ? 0 : kRowMaxRows * kRowTaps * ROWS * 4); }
    __host__ __device__ static int off_halopos(int halo) { return off_haloaddr() + pixels(halo) * 8; }
    __host__ __device__ static int off_raw(int halo) { return off_halopos(halo) + (kSparse ? pixels(halo) * 4 : 0); }
    __host__ __device__ static int off_a(int halo) { return off_raw(halo) + (kPrunes ? 2 * kRawSlot : 0); }
    __host__ __device__ static int a_bytes(int halo, int npad) { return kSparse ? 2 * plane_a(npad) : pixels(halo) * kAPitch; }
    __host__ __device__ static int off_meta(int halo, int npad) { return off_a(halo) + 2 * a_bytes(halo, npad); }
    __host__ __device__ static int meta_bytes(int npad) { return kSparse ? 2 * plane_m(npad) : 0; }
    __host__ __device__ static int total(int halo, int npad) {
        const int loop = off_meta(halo, npad) + 2 * meta_bytes(npad);
        const int out = off_out() + ROWS * kOutPitch;
        return loop > out ? loop : out;
    }
};

template <int BN, int MODE, int M, int RK, int ROWS>
__global__ void __launch_bounds__(512) bwd_row(const RowParams p) {
    using L = RowLayout<BN, MODE, ROWS>;
    static_assert(ROWS == 512 || ROWS == 256, "rows of a workgroup tile");
    constexpr bool SPARSE = MODE == 2;
    constexpr bool PRUNES = MODE != 0;
    constexpr int KC = kRowKC;
    constexpr int TS = kRowTaps;
    constexpr int WAVES_N = BN / 64;
    constexpr int WAVES_M = 8 / WAVES_N;
    constexpr int WM = ROWS / WAVES_M;
    constexpr int TM = WM / 32;
    constexpr int TN = 2;
    constexpr int KSTEP = SPARSE ? 32 : 16;
    constexpr int NKS = KC / KSTEP;
    constexpr int NQ = TS * NKS;                // k-steps per stage
    constexpr int CPR = BN / 8;                 // 16-byte columns per W row
    // Swizzle of the W slab: the 16-byte column of row r sits at column ^ (WSW * (r & 3)).  One pass of a transpose read
    // takes rows r .. r+3 and four columns of each; with 64 banks of 4 bytes a row of 256 bytes or more starts at bank 0,
    // so the four rows must land in four different quarters of the 256-byte bank window (WSW = 4); a 128-byte row
    // alternates between the two halves of the window by itself and only needs its halves told apart (WSW = 2).
    constexpr int WSW = BN >= 128 ? 4 : 2;
    constexpr int RPU = 1024 / L::kWRow;        // W rows per copy unit
    constexpr int WU = L::kWUnits;

    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDS unsigned char* smem = (SDGP_LDS unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- which tile: consecutive logical ids stay on one XCD (workgroups are dealt round-robin over 8 XCDs)
    int lid = blockIdx.x;
    {
        const int per = p.nblocks >> 3;
        if (lid < (per << 3)) lid = (lid & 7) * per + (lid >> 3);
    }
    const int ntile = lid % p.ntiles_n;
    const int mtile = lid / p.ntiles_n;
    const int tw_i = mtile % p.tiles_w;
    const int th_i = (mtile / p.tiles_w) % p.tiles_h;
    const int tb_i = mtile / (p.tiles_w * p.tiles_h);
    const int b0 = tb_i * p.TB, hh0 = th_i * p.TH, ww0 = tw_i * p.TW;
    const int n0 = ntile * BN;
    const int tile_rows = p.TB * p.TH * p.TW;
    const int tile_hw = p.TH * p.TW;
    const int R = p.R;
    // halo: the gradient pixels the tile's taps reach, clipped to the image (tap (r, s) reads pixel (h + pad - r, w + pad - s))
    const int py0 = max(0, hh0 + p.pad - (R - 1)), py1 = min(p.P, hh0 + p.TH + p.pad);
    const int qx0 = max(0, ww0 + p.pad - (TS - 1)), qx1 = min(p.Q, ww0 + p.TW + p.pad);
    const int HTH = py1 - py0, HTW = qx1 - qx0;
    const int halo_hw = HTH * HTW;
    const int nhalo = p.TB * halo_hw;
    const int nunits = (nhalo + 15) >> 4;
    const int nchunks = p.C_out / KC;
    const int nstages = R * nchunks;
    // every workgroup walks the chunks and the filter rows in its own rotation: the sum does not care, and the
    // workgroups of an XCD then ask its L2 for different W slabs at a given moment
    const int c_rot = mtile % nchunks, r_rot = (mtile / nchunks) % R;

    SDGP_LDS int* rowpix = (SDGP_LDS int*)(smem + L::off_rowpix());
    typedef unsigned long long u64_t;
    SDGP_LDS u64_t* haloaddr = (SDGP_LDS u64_t*)(smem + L::off_haloaddr());
    SDGP_LDS uint32_t* atab = (SDGP_LDS uint32_t*)(smem + L::off_atab());
    const uint32_t off_a = (uint32_t)L::off_a(p.halo_max), a_buf_bytes = (uint32_t)L::a_bytes(p.halo_max, p.npad);
    const uint32_t off_meta = (uint32_t)L::off_meta(p.halo_max, p.npad), meta_buf_bytes = (uint32_t)L::meta_bytes(p.npad);
    const uint32_t off_raw = (uint32_t)L::off_raw(p.halo_max);
    const uint32_t zero_pix = (uint32_t)L::zero_pixel(p.halo_max);
    // compressed halo: the zero-padded grid of the positions the tile's taps reach, image borders included
    // (tap (r, s) of tile pixel (hl, wl) reads grid position (hl + R - 1 - r, wl + 2 - s)); positions outside the
    // gradient stay zero, so a tap is a constant offset from a row's base position and needs no table
    const int GH = p.TH + R - 1, GW = p.TW + TS - 1;
    const int g_p0 = hh0 + p.pad - (R - 1), g_q0 = ww0 + p.pad - (TS - 1);  // gradient pixel of grid position (0, 0)
    const uint32_t plane_a = (uint32_t)L::plane_a(p.npad), plane_m = (uint32_t)L::plane_m(p.npad);
    SDGP_LDS uint32_t* halopos = (SDGP_LDS uint32_t*)(smem + L::off_halopos(p.halo_max));
    const uint16_t* const gdO = p.dO;
    const unsigned char* const gWb = reinterpret_cast<const unsigned char*>(p.W);

    // ---- tables (one row of the tile per thread)
    //   rowpix[m]        output pixel of tile row m (-1: none)
    //   atab[tap][m]     byte offset, inside a halo buffer, of the gradient pixel that tap `tap` of row m reads
    //                    (dense: with the pixel's swizzle; the zero pixel when the tap falls outside the image)
    //   haloaddr[hp]     address of channel 0 of halo pixel hp
    // The address table of the halo comes first: the first copies need nothing else and fly while the rest is built.
    for (int hp = tid; hp < L::pad16(nhalo); hp += 512) {
        size_t gp = 0;  // positions past the halo (tail of the last copy unit) copy pixel 0; nobody reads them
        if (hp < nhalo) {
            const int tb = hp / halo_hw, rem = hp % halo_hw;
            const int b = min(b0 + tb, p.B - 1);  // images past the batch: valid memory, rows never stored
            const int py = py0 + rem / HTW, qx = qx0 + rem % HTW;
            gp = ((size_t)b * p.P + py) * p.Q + qx;
            if constexpr (SPARSE) halopos[hp] = (uint32_t)((tb * GH + (py - g_p0)) * GW + (qx - g_q0));
        }
        haloaddr[hp] = (u64_t)(uintptr_t)(gdO + gp * p.C_out);
    }
    auto build_row_tables = [&]() {
      if (tid < ROWS) {
        const int m = tid;
        int pix = -1, rowbase = 0, h = 0, w = 0;
        bool live = false;
        if (m < tile_rows) {
            const int tb = m / tile_hw, rem = m % tile_hw;
            h = hh0 + rem / p.TW, w = ww0 + rem % p.TW;
            if (b0 + tb < p.B && h < p.H && w < p.Wd) {
                live = true;
                pix = ((b0 + tb) * p.H + h) * p.Wd + w;
                rowbase = (tb * HTH + (h - py0)) * HTW + (w - qx0);
            }
        }
        rowpix[m] = pix;
        if constexpr (!SPARSE) {
            for (int r = 0; r < R; ++r)
                for (int sx = 0; sx < TS; ++sx) {
                    const int pp = h + p.pad - r, qq = w + p.pad - sx;
                    const bool inside = live && pp >= 0 && pp < p.P && qq >= 0 && qq < p.Q;
                    const uint32_t hp = inside ? (uint32_t)(rowbase + (p.pad - r) * HTW + (p.pad - sx)) : zero_pix;
                    atab[(r * TS + sx) * ROWS + m] = hp * 64u + (((hp >> 2) & 3u) << 4);
                }
        }
      }
      if constexpr (!SPARSE) {
        if (tid < 32) {
            // the zero pixel of both halo buffers
            const uint32_t buf = tid >> 4, i = tid & 15;
            *(SDGP_LDS uint32_t*)(smem + off_a + buf * a_buf_bytes + zero_pix * L::kAPitch + i * 4) = 0u;
        }
      } else {
        // both compressed buffers start as zeros: values 0 (and positions 0) wherever the ranking never writes
        const u32x4_t z = {0u, 0u, 0u, 0u};
        const uint32_t bytes = 2u * a_buf_bytes + 2u * meta_buf_bytes;  // the value planes and the position planes are adjacent
        for (uint32_t o = (uint32_t)tid * 16u; o < bytes; o += 512u * 16u) *(SDGP_LDS u32x4_t*)(smem + off_a + o) = z;
      }
    };

    // ---- copies
    uint32_t w_voff;  // this lane's byte offset inside a slab's source: the wavefront copies unit (wave % WU) of a slab
    {
        const int row = (wave % WU) * RPU + lane / CPR;
        const int lchunk = (lane % CPR) ^ (WSW * (row & 3));
        int col = n0 + lchunk * 8;
        if (col > p.C_in - 8) col = p.C_in - 8;  // columns past C_in feed accumulators that are never stored
        w_voff = (uint32_t)(row * p.w_row + col) * 2u;
    }
    const uint32_t tapB = (uint32_t)p.C_in * 2u;                    // bytes between the slabs of consecutive taps
    const uint32_t chunkB = (uint32_t)KC * (uint32_t)p.w_row * 2u;  // ... of consecutive chunks
    // the three slabs of (physical chunk pc, physical filter row pr) into ring set `set`
    auto copy_w_set = [&](int pc, int pr, int set) {
        for (int i = wave; i < TS * WU; i += 8) {
            const int j = i / WU;
            lds_copy16(gWb + ((size_t)pc * chunkB + (size_t)(pr * TS + j) * tapB), w_voff,
                        smem_base + L::off_w() + (uint32_t)set * L::kWSet + (uint32_t)j * L::kWSlab + (uint32_t)(wave % WU) * 1024u);
        }
    };
    // 16-byte column a lane copies: LDS position (lane & 3) of pixel (lane >> 2) holds the swizzled source column
    const uint32_t c16_halo = PRUNES ? (uint32_t)(((lane & 3) ^ ((lane >> 4) & 1)) * 16)
                                     : (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) * 16);
    const uint32_t haloaddr_lane = (uint32_t)L::off_haloaddr() + (uint32_t)(lane >> 2) * 8u;
    // unit u of the halo, channels at byte offset src_off of every pixel, to LDS address dst
    auto copy_halo = [&](int u, uint32_t src_off, uint32_t dst) {
        const u64_t a = *(SDGP_LDS u64_t*)(smem + haloaddr_lane + (uint32_t)u * 128u);
        lds_copy16(reinterpret_cast<const void*>((uintptr_t)(a + (u64_t)(c16_halo + src_off))), dst);
    };
    // up to two units per wavefront of the share [u0, u0 + cnt) of a chunk's halo; unit u0 + i lands at dst0 + i KB
    auto copy_halo_share = [&](int u0, int cnt, int pc, uint32_t dst0) {
        for (int i = wave; i < cnt; i += 8) copy_halo(u0 + i, (uint32_t)pc * (KC * 2), dst0 + (uint32_t)i * 1024u);
    };

    // rank / prune / compress 64 items (pixel, 16-channel half) of a raw share into a halo buffer (Sec. III-B)
    auto prune_items = [&](int item0, int nitems, int u0, uint32_t raw, uint32_t abuf, uint32_t mbuf, uint32_t chan0) {
        if constexpr (PRUNES && !SPARSE) {
            // any n of m (m up to 32): the pruned pixels are stored dense, zeros in the dropped positions, in the
            // layout the dense matrix instruction reads.  A 32-group is the whole chunk of a pixel: the lane of its
            // first half takes it.
            constexpr int IC = M > 16 ? 32 : 16;  // channels per item
            const int item = item0 + lane;
            const int j = item >> 5, px = (item >> 1) & 15, part = item & 1;
            const int hp = (u0 + j) * 16 + px;
            if (item < nitems && hp < nhalo && (IC == 16 || part == 0)) {
                SDGP_LDS unsigned char* src = smem + raw + j * 1024 + px * 64;
                SDGP_LDS unsigned char* dst = smem + abuf + hp * 64;
                const int sw = (px >> 2) & 1, sw2 = (hp >> 2) & 3;
                if constexpr (RK != kRandom && (M == 16 || M == 32)) {
                    // one group per item, magnitude keys: the packed 16-bit ranker (ranker.h), no unpacking
                    uint32_t wv[IC / 2], ov[IC / 2];
#pragma unroll
                    for (int g = 0; g < IC / 8; ++g) {
                        const u32x4_t v = *(SDGP_LDS u32x4_t*)(src + (((part * 2 + g) ^ sw) * 16));
                        wv[4 * g] = v[0], wv[4 * g + 1] = v[1], wv[4 * g + 2] = v[2], wv[4 * g + 3] = v[3];
                    }
                    prune_packed<M, RK>(wv, p.n, ov);
#pragma unroll
                    for (int g = 0; g < IC / 8; ++g) {
                        const u32x4_t x = {ov[4 * g], ov[4 * g + 1], ov[4 * g + 2], ov[4 * g + 3]};
                        *(SDGP_LDS u32x4_t*)(dst + (((part * 2 + g) ^ sw2) << 4)) = x;
                    }
                    return;
                }
                uint32_t rawv[IC], out[IC];
#pragma unroll
                for (int g = 0; g < IC / 8; ++g) {
                    const u32x4_t v = *(SDGP_LDS u32x4_t*)(src + (((part * 2 + g) ^ sw) * 16));
#pragma unroll
                    for (int x = 0; x < 4; ++x) rawv[g * 8 + 2 * x] = v[x] & 0xFFFFu, rawv[g * 8 + 2 * x + 1] = v[x] >> 16;
                }
                uint64_t e0 = 0;
                if constexpr (RK == kRandom)
                    e0 = ((uint64_t)(haloaddr[hp] - (u64_t)(uintptr_t)gdO) >> 1) + (uint64_t)(chan0 + part * 16);
#pragma unroll
                for (int g = 0; g < IC / M; ++g) {
                    uint32_t rr[M], o[M];
                    bool kk[M];
#pragma unroll
                    for (int jj = 0; jj < M; ++jj) rr[jj] = rawv[g * M + jj];
                    const uint64_t eg = e0 + (uint64_t)(g * M);
                    prune_group<kBF16, M, RK, false>(rr, p.n, hash_row(p.mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
                    for (int jj = 0; jj < M; ++jj) out[g * M + jj] = o[jj];
                }
#pragma unroll
                for (int g = 0; g < IC / 8; ++g) {
                    const u32x4_t x = {out[g * 8] | (out[g * 8 + 1] << 16), out[g * 8 + 2] | (out[g * 8 + 3] << 16),
                                       out[g * 8 + 4] | (out[g * 8 + 5] << 16), out[g * 8 + 6] | (out[g * 8 + 7] << 16)};
                    *(SDGP_LDS u32x4_t*)(dst + (((part * 2 + g) ^ sw2) << 4)) = x;
                }
            }
        }
        if constexpr (SPARSE) {
            const int item = item0 + lane;
            const int j = item >> 5, px = (item >> 1) & 15, part = item & 1;
            const int hp = (u0 + j) * 16 + px;
            if (item < nitems && hp < nhalo) {
                SDGP_LDS unsigned char* src = smem + raw + j * 1024 + px * 64;
                const int sw = (px >> 2) & 1;
                u32x4_t v[2];
                v[0] = *(SDGP_LDS u32x4_t*)(src + (((2 * part) ^ sw) * 16));
                v[1] = *(SDGP_LDS u32x4_t*)(src + (((2 * part + 1) ^ sw) * 16));
                uint64_t e0 = 0;
                if constexpr (RK == kRandom)
                    e0 = ((uint64_t)(haloaddr[hp] - (u64_t)(uintptr_t)gdO) >> 1) + (uint64_t)(chan0 + part * 16);
                uint32_t packed[4], meta;
                prune16_compressed<M, RK>(v, p.n, p.mix, e0, packed, meta);
                const u32x4_t x = {packed[0], packed[1], packed[2], packed[3]};
                const uint32_t pos = halopos[hp];
                *(SDGP_LDS u32x4_t*)(smem + abuf + (uint32_t)part * plane_a + pos * 16u) = x;
                *(SDGP_LDS uint16_t*)(smem + mbuf + (uint32_t)part * plane_m + pos * 2u) = (uint16_t)meta;
            }
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int u = 0; u < TN; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.0f;

    __syncthreads();  // halo address table visible

    // ---- prologue: the first chunk's halo, the first stage's slabs, the raw share the first stage prunes; the row
    // tables are built while the first copies are in flight
    const int ups = p.ups;
    const int pc1 = c_rot + 1 == nchunks ? 0 : c_rot + 1;  // physical chunk of logical chunk 1
    copy_w_set(c_rot, r_rot, 0);
    if constexpr (!PRUNES) {
        for (int u = wave; u < nunits; u += 8) copy_halo(u, (uint32_t)c_rot * (KC * 2), smem_base + off_a + u * 1024);
        build_row_tables();
    } else {
        // rounds of 16 units through the two raw slots: round r + 1 is in flight while round r is ranked
        const int rounds = (nunits + 15) / 16;
        copy_halo_share(0, min(16, nunits), c_rot, smem_base + off_raw);
        build_row_tables();
        for (int r = 0; r < rounds; ++r) {
            wait_lds_copies<0>();
            __syncthreads();  // round r has landed; everybody is done with the slot round r + 1 goes into
            if (r + 1 < rounds)
                copy_halo_share((r + 1) * 16, min(16, nunits - (r + 1) * 16), c_rot,
                                smem_base + off_raw + (uint32_t)((r + 1) & 1) * L::kRawSlot);
            prune_items(wave * 64, 512, r * 16, off_raw + (uint32_t)(r & 1) * L::kRawSlot, off_a, off_meta, (uint32_t)c_rot * KC);
        }
        __syncthreads();  // the last round is ranked: raw slot 0 is free again
        if (nchunks > 1) copy_halo_share(0, min(ups, nunits), pc1, smem_base + off_raw);
    }
    wait_lds_copies<0>();
    __syncthreads();

    // ---- fragments
    uint32_t b_lane[TN];  // transpose reads from the swizzled slab, one lane address per 32-column tile
#pragma unroll
    for (int u = 0; u < TN; ++u) {
        const int L16 = lane & 15;
        const int chunk = 8 * wn + 4 * u + 2 * ((lane >> 4) & 1) + ((L16 & 3) >> 1);
        b_lane[u] = (uint32_t)(L::off_w() + (8 * (lane >> 5) + (L16 >> 2)) * L::kWRow + ((chunk ^ (WSW * (L16 >> 2))) * 16) +
                               (L16 & 1) * 8);
    }
    struct Frags {
        u32x4_t a[TM];
        int meta[TM];
        typename std::conditional<SPARSE, bf16x16_t, bf16x8_t>::type b[TN];
    };
    const uint32_t half = (uint32_t)(lane >> 5);
    const uint32_t atab_lane = (uint32_t)L::off_atab() + (uint32_t)(wm * WM + (lane & 31)) * 4u;
    uint32_t a_ent[TM];    // table entries of the tap whose fragments are being requested
    uint32_t a_ent_n[TM];  // ... of the tap after it (requested early)
    auto read_entries = [&](int tap) {
#pragma unroll
        for (int t = 0; t < TM; ++t) a_ent_n[t] = *(SDGP_LDS uint32_t*)(smem + atab_lane + (uint32_t)tap * (ROWS * 4) + t * 128);
    };
    auto take_entries = [&]() {
#pragma unroll
        for (int t = 0; t < TM; ++t) a_ent[t] = a_ent_n[t];
    };
    const uint32_t a_k0 = half << 4;
    // compressed halo: per row tile the lane's byte offsets into the value and position planes of its half of the
    // chunk, at the grid position of the row's LAST tap of filter row 0 (tap s of filter row r sits (TS - 1 - s)
    // positions after it and r grid rows before); a_stage / m_stage add the buffer and the filter row once per stage
    uint32_t lane_a[TM], lane_m[TM], a_stage[TM], m_stage[TM];
    if constexpr (SPARSE) {
#pragma unroll
        for (int t = 0; t < TM; ++t) {
            const int m = wm * WM + t * 32 + (lane & 31);
            int pos = (R - 1) * GW;  // rows without an output pixel read image 0's first grid positions: valid memory
            if (m < tile_rows) {
                const int tb = m / tile_hw, rem = m % tile_hw;
                const int hl = rem / p.TW, wl = rem % p.TW;
                if (b0 + tb < p.B && hh0 + hl < p.H && ww0 + wl < p.Wd) pos = (tb * GH + hl + R - 1) * GW + wl;
            }
            lane_a[t] = half * plane_a + (uint32_t)pos * 16u;
            lane_m[t] = half * plane_m + (uint32_t)pos * 2u;
        }
    }
    auto set_stage = [&](uint32_t abuf, uint32_t mbuf, int frow) {
        if constexpr (SPARSE) {
            const uint32_t back = (uint32_t)(frow * GW);
#pragma unroll
            for (int t = 0; t < TM; ++t) a_stage[t] = lane_a[t] + (abuf - back * 16u), m_stage[t] = lane_m[t] + (mbuf - back * 2u);
        }
    };
    // tap: position in the filter row (compressed halo); ks: k-step inside the chunk (table-driven halo)
    auto load_a = [&](Frags& f, int t, uint32_t abuf, int tap, int ks) {
        if constexpr (SPARSE) {
            f.a[t] = *(SDGP_LDS u32x4_t*)(smem + a_stage[t] + (TS - 1 - tap) * 16);
            f.meta[t] = *(SDGP_LDS uint16_t*)(smem + m_stage[t] + (TS - 1 - tap) * 2);
        } else {
            f.a[t] = *(SDGP_LDS u32x4_t*)(smem + ((a_ent[t] ^ (a_k0 | (uint32_t)(ks * 32))) + abuf));
        }
    };
    auto load_b = [&](Frags& f, int u, uint32_t slab_off, int ks) {
        SDGP_LDS unsigned char* wb = smem + b_lane[u] + slab_off;
        if constexpr (SPARSE) {
            s16x4_t q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SDGP_LDS s16x4_t*)(wb + ((i >> 1) * 16 + (i & 1) * 4) * L::kWRow));
            typedef short s16x16_t __attribute__((ext_vector_type(16)));
            const s16x16_t all = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3],
                                  q[2][0], q[2][1], q[2][2], q[2][3], q[3][0], q[3][1], q[3][2], q[3][3]};
            f.b[u] = __builtin_bit_cast(bf16x16_t, all);
        } else {
            s16x4_t q[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SDGP_LDS s16x4_t*)(wb + (ks * 16 + i * 4) * L::kWRow));
            typedef short s16x8_t __attribute__((ext_vector_type(8)));
            const s16x8_t all = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3]};
            f.b[u] = __builtin_bit_cast(bf16x8_t, all);
        }
    };
    auto mma_one = [&](const Frags& f, int t, int u) {
        const bf16x8_t a = __builtin_bit_cast(bf16x8_t, f.a[t]);
        if constexpr (SPARSE)
            acc[t][u] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, f.b[u], acc[t][u], f.meta[t], 0, 0);
        else
            acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, f.b[u], acc[t][u], 0, 0, 0);
    };

    // ---- main loop: one stage = (chunk, filter row).  A matrix instruction occupies the pipe for 32 cycles and a
    // wavefront issues in order, so the requests for the next k-step's fragments and the stage's copies are cut into
    // pieces of a few instructions and placed between the matrix instructions.
    int c = 0, r = 0;                                      // logical chunk and filter row
    int pc = c_rot, pr = r_rot;                            // physical
    uint32_t abuf = off_a, mbuf = off_meta;               // halo buffer of the current chunk
    uint32_t abuf_other = off_a + a_buf_bytes, mbuf_other = off_meta + meta_buf_bytes;
    constexpr int GAPS = TM * TN;
    constexpr int APIECES = (TM + 1) / 2;
    Frags fr[2];
    auto stage = [&](Frags& f0, Frags& f1, int x) {
        const uint32_t set_off = (uint32_t)(x & 1) * L::kWSet;
        const int pc_next = pc + 1 == nchunks ? 0 : pc + 1;
        const bool row_last = r + 1 == R;
        // next stage
        const int nr = row_last ? 0 : r + 1, nc = row_last ? c + 1 : c;
        const int npr = pr + 1 == R ? 0 : pr + 1;
        const int npc = row_last ? pc_next : pc;
        const bool more = x + 1 < nstages;
        // first k-step: nothing of this stage was requested before the barrier except the table entries
        if constexpr (SPARSE) {
            set_stage(abuf, mbuf, pr);
        } else {
            read_entries(pr * TS);
            take_entries();
        }
#pragma unroll
        for (int t = 0; t < TM; ++t) load_a(f0, t, abuf, 0, 0);
#pragma unroll
        for (int u = 0; u < TN; ++u) load_b(f0, u, set_off, 0);
        // share r of the next chunk's halo: one item per lane of the whole workgroup.  The two wavefronts of a SIMD
        // (w and w + 4) rank at different times -- one before the stage's first k-step, the other after it -- so
        // that one's vector work runs under the other's matrix instructions.
        auto prune_share = [&]() {
            if constexpr (PRUNES) {
                if (c + 1 < nchunks) {
                    const int u0 = r * ups;
                    const int cnt = min(ups, nunits - u0);
                    if (cnt > 0)
                        prune_items(wave * 64, cnt * 32, u0, off_raw + (uint32_t)(x & 1) * L::kRawSlot, abuf_other, mbuf_other,
                                    (uint32_t)pc_next * KC);
                }
            }
        };
        if (wave < 4) prune_share();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            Frags& cur = (q & 1) ? f1 : f0;
            Frags& nxt = (q & 1) ? f0 : f1;
            const int tap = q / NKS, ks = q % NKS;
            const bool has_next = q + 1 < NQ;
            const int ntap = (q + 1) / NKS, nks = (q + 1) % NKS;
            const bool entries_now = has_next && ks == 0 && tap + 1 < TS && NKS > 1;   // read the next tap's entries early
            const bool new_tap = has_next && ntap != tap;
            if (q == 1) {
                if (wave >= 4) prune_share();
                __builtin_amdgcn_sched_barrier(0);
            }
            // pieces: 0 table entries; 1..APIECES A fragments (two row tiles each); then TN B fragments;
            // in the first k-step also 3 copy pieces
            const int npieces = 1 + APIECES + TN + (q == 0 ? 3 : 0);
            auto piece = [&](int i) {
                if (i == 0) {
                    if constexpr (!SPARSE) {
                        if (entries_now) read_entries(pr * TS + tap + 1);
                        if (NKS == 1 && new_tap) read_entries(pr * TS + ntap);
                    }
                } else if (i <= APIECES) {
                    if (has_next) {
                        if constexpr (!SPARSE) {
                            if (i == 1 && new_tap) take_entries();
                        }
                        const int t0 = 2 * (i - 1);
                        load_a(nxt, t0, abuf, ntap, nks);
                        if (t0 + 1 < TM) load_a(nxt, t0 + 1, abuf, ntap, nks);
                    }
                } else if (i <= APIECES + TN) {
                    if (has_next) load_b(nxt, i - APIECES - 1, set_off + (uint32_t)ntap * L::kWSlab, nks);
                } else if (i == APIECES + TN + 1) {
                    if (more) copy_w_set(npc, npr, (x + 1) & 1);
                } else if (i == APIECES + TN + 2) {
                    if constexpr (!PRUNES) {
                        // dense: share r of the next chunk's halo straight into the other buffer
                        if (c + 1 < nchunks) {
                            const int u0 = r * ups;
                            copy_halo_share(u0, min(ups, nunits - u0), pc_next, smem_base + abuf_other + (uint32_t)u0 * 1024u);
                        }
                    } else {
                        // pruning: the raw share that the next stage ranks (share nr of the chunk after the next stage's)
                        if (more && nc + 1 < nchunks) {
                            const int u0 = nr * ups;
                            const int fpc = npc + 1 == nchunks ? 0 : npc + 1;
                            copy_halo_share(u0, min(ups, nunits - u0), fpc, smem_base + off_raw + (uint32_t)((x + 1) & 1) * L::kRawSlot);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            int done = 0;
#pragma unroll
            for (int g = 0; g < GAPS; ++g) {
                mma_one(cur, g / TN, g % TN);
                __builtin_amdgcn_sched_barrier(0);
                const int upto = ((g + 1) * npieces + GAPS - 1) / GAPS;
                for (; done < upto && done < npieces; ++done) piece(done);
            }
        }
        wait_lds_copies<0>();
        __syncthreads();  // never optional: the epilogue reuses the tables' LDS as soon as a wavefront leaves the loop
        if (row_last) {
            r = 0, ++c, pc = pc_next;
            const uint32_t xa = abuf; abuf = abuf_other; abuf_other = xa;
            const uint32_t xm = mbuf; mbuf = mbuf_other; mbuf_other = xm;
        } else {
            ++r;
        }
        pr = npr;
    };
    if constexpr (NQ % 2 == 0) {
        for (int x = 0; x < nstages; ++x) stage(fr[0], fr[1], x);
    } else {
        int x = 0;
        for (; x + 1 < nstages; x += 2) {
            stage(fr[0], fr[1], x);
            stage(fr[1], fr[0], x + 1);
        }
        if (x < nstages) stage(fr[0], fr[1], x);
    }

    // ---- epilogue: fp32 -> bf16 (RNE) into LDS, then whole pixel rows with 16-byte stores
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    SDGP_LDS unsigned char* outb = smem + L::off_out();
#pragma unroll
    for (int tt = 0; tt < TM; ++tt)
#pragma unroll
        for (int u = 0; u < TN; ++u)
#pragma unroll
            for (int rr = 0; rr < 16; rr += 2) {
                // registers rr and rr + 1 are two consecutive rows of one column
                const int m = wm * WM + tt * 32 + 8 * (rr >> 2) + 4 * (lane >> 5) + (rr & 3);
                const int col = wn * 64 + u * 32 + (lane & 31);
                const f32x2_t v = {acc[tt][u][rr], acc[tt][u][rr + 1]};
                const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
                *(SDGP_LDS uint16_t*)(outb + m * L::kOutPitch + col * 2) = (uint16_t)pk;
                *(SDGP_LDS uint16_t*)(outb + (m + 1) * L::kOutPitch + col * 2) = (uint16_t)(pk >> 16);
            }
    __syncthreads();
#pragma unroll 4
    for (int idx = tid; idx < ROWS * CPR; idx += 512) {
        const int m = idx / CPR, cc = idx % CPR;
        const int pix = rowpix[m];
        if (pix >= 0 && n0 + cc * 8 < p.C_in) {
            const u32x4_t v = *(SDGP_LDS u32x4_t*)(outb + m * L::kOutPitch + cc * 16);
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p.dD + (size_t)pix * p.C_in + n0 + cc * 8));
        }
    }
}

}  // namespace sdgp
