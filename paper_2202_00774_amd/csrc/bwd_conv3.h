// Asynchronous-copy variant of the tiled backward-data kernel for stride-1 filters with at
// least four taps (3x3, 5x5, 7x7): the layers where the product is bound by the matrix cores.
//
// Same decomposition as bwd_tiled.h (256-pixel x BN-column tile per workgroup, 64-channel
// chunks, one barrier per (chunk, tap) stage, 4 consumer + 4 producer wavefronts), but every
// byte that comes from global memory is moved by direct-to-LDS loads
// (global_load_lds_dwordx4: lane i of a wavefront writes 16 bytes at LDS base + 16*i).
// They need no destination registers, so a wavefront keeps three stages of copies in
// flight and waits with an explicit counter: each producer wavefront issues exactly
// kPer copies per stage, hence "all but the last kPer copies have landed" means "everything
// issued before this stage is in LDS".
//
//   * W slabs (64 x BN, the layout W has in memory) go into a ring of 4 slots, requested
//     three stages ahead.  Rows are unpadded; the 16-byte chunk index is XOR-swizzled with
//     2*(row & 3) on the global-address side so the transpose reads that build B fragments
//     hit distinct banks.
//   * Dense (MODE 0): the gradient halo of the next chunk is copied straight into the other
//     halo buffer (128 bytes per pixel, chunk index swizzled with (pixel >> 1) & 7).
//   * Sparse (MODE 2): the raw halo streams through a ring of 4 batches (64 pixels each); the
//     producers read a batch back from LDS three stages after requesting it, rank / prune /
//     compress it (Sec. III-B) and write the compressed halo buffer of the next chunk.
//   * Pixels outside the image are copied from a 128-byte row of zeros in device memory, so the
//     padding needs no arithmetic anywhere.
#pragma once

#include <type_traits>

#include "bwd_tiled.h"

namespace sdgp {

struct Conv3Params {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    int B, P, Q, C_out, C_in;       // stride 1: dD is [B, H, Wd, C_in] with H, Wd below
    int H, Wd;
    int w_row;                      // elements per W row: R*S*C_in
    int n;
    uint32_t mix;
    int TB, TH, TW;                 // tile: TB images x TH x TW pixels (<= 256)
    int tiles_h, tiles_w;
    int HTH, HTW, dpmin, dqmin;     // halo
    int nhalo, nunits;              // halo pixels, 8-pixel copy units
    int ntaps;
    int ntiles_n, nblocks;
    TapEntry taps[kMaxTaps];
};

constexpr int kC3KC = 64;           // reduction channels per chunk
constexpr int kC3Slots = 4;         // W ring
constexpr int kC3RawSlots = 4;      // raw halo ring (sparse)
constexpr int kC3UnitsPerStep = 8;  // halo copy units (8 pixels x 128 B) per stage
#ifndef SDGP_C3_CONSUMERS
#define SDGP_C3_CONSUMERS 8
#endif
constexpr int kC3Consumers = SDGP_C3_CONSUMERS;  // matrix wavefronts per workgroup (the producers follow them)
// Producer wavefronts: copies alone need few instructions, ranking a halo needs many, and one wavefront issues
// at most one instruction every four cycles -- so the pruning kernels get two producers per SIMD.
__host__ __device__ constexpr int conv3_producers(int mode) { return mode == 2 ? 8 : 4; }
__host__ __device__ constexpr int conv3_threads(int mode) { return (kC3Consumers + conv3_producers(mode)) * 64; }

template <int BN, int MODE>
struct Conv3Layout {
    static constexpr bool kSparse = MODE == 2;
    static constexpr int kWRow = BN * 2;
    static constexpr int kWSlab = kC3KC * kWRow;
    static constexpr int kAPitch = kSparse ? 80 : 128;
    static constexpr int kMetaPitch = 8;
    static constexpr int kRawSlot = kC3UnitsPerStep * 1024;
    __host__ __device__ static int pad8(int halo) { return (halo + 7) & ~7; }
    __host__ __device__ static int off_w() { return 0; }
    __host__ __device__ static int off_sink() { return kC3Slots * kWSlab; }
    __host__ __device__ static int off_rowpix() { return off_sink() + 1024; }
    __host__ __device__ static int off_halopix(int) { return off_rowpix() + kTileRows * 4; }
    __host__ __device__ static int off_raw_h(int halo) { return off_halopix(halo) + pad8(halo) * 8; }
    __host__ __device__ static int off_a_h(int halo) { return off_raw_h(halo) + (kSparse ? kC3RawSlots * kRawSlot : 0); }
    __host__ __device__ static int a_bytes(int halo) { return pad8(halo) * kAPitch; }
    __host__ __device__ static int off_meta(int halo) { return off_a_h(halo) + 2 * a_bytes(halo); }
    __host__ __device__ static int meta_bytes(int halo) { return kSparse ? pad8(halo) * kMetaPitch : 0; }
    __host__ __device__ static int total(int halo) { return off_meta(halo) + 2 * meta_bytes(halo); }
};

// A row of zeros in device memory: the source of halo pixels that lie outside the image.  Long enough for every
// chunk offset of the widest gradient the kernel takes, so those pixels need no special case when a chunk advances.
constexpr int kC3MaxCout = 4096;
__device__ const uint32_t kZeroRow[kC3MaxCout / 2 + 32] = {0};

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_base + 16*i.
// The compiler does not see this as a memory instruction; callers count copies and wait with wait_copies.
__device__ __forceinline__ void copy16_to_lds(const void* gptr, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);  // wave-uniform by construction
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(gptr) : "memory");
}

// Same, with the address split into a wave-uniform base and a 32-bit byte offset per lane (no address arithmetic on
// the vector unit when only the base moves).
__device__ __forceinline__ void copy16_to_lds(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}

// Waits until at most N of this wavefront's vector-memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wait_copies() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

template <int BN, int MODE, int M, int RK>
__global__ void __launch_bounds__(conv3_threads(MODE)) bwd_conv3(const Conv3Params p) {
    using L = Conv3Layout<BN, MODE>;
    constexpr bool SPARSE = MODE == 2;
    constexpr int KC = kC3KC;
    // 8 consumer wavefronts (two per SIMD, so one wave's LDS reads and address arithmetic issue while the
    // other's matrix instructions execute) and 4 producer wavefronts
    constexpr int WAVES_N = BN / 64;
    constexpr int WAVES_M = kC3Consumers / WAVES_N;
    constexpr int WM = kTileRows / WAVES_M;
    constexpr int TM = WM / 32;
    constexpr int TN = 2;
    constexpr int KSTEP = SPARSE ? 32 : 16;
    constexpr int NKS = KC / KSTEP;
    constexpr int W_UNITS = L::kWSlab / 1024;          // 1 KB copy units per slab
    constexpr int NP = conv3_producers(MODE);          // producer wavefronts
    constexpr int WPW = W_UNITS / NP;                  // per producer wavefront
    constexpr int HPW = kC3UnitsPerStep / NP;          // halo units per producer wavefront per stage
    static_assert(WPW >= 1 && HPW >= 1 && WPW * NP == W_UNITS && HPW * NP == kC3UnitsPerStep, "copy units divide evenly");
    constexpr int kPer = WPW + HPW;                    // copies a producer wavefront issues per stage
    constexpr int CPR = BN / 8;                        // 16-byte chunks per W row
    // Swizzle of the W slab: the 16-byte column of row r sits at column ^ (WSW * (r & 3)).  One pass of a transpose read
    // takes rows r .. r+3 and four columns of each; with 64 banks of 4 bytes a row of 256 bytes or more starts at bank 0,
    // so the four rows must land in four different quarters of the 256-byte bank window (WSW = 4); a 128-byte row
    // alternates between the two halves of the window by itself and only needs its halves told apart (WSW = 2).
    constexpr int WSW = BN >= 128 ? 4 : 2;
    constexpr int RPU = 1024 / L::kWRow;               // W rows per copy unit

    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDS unsigned char* smem = (SDGP_LDS unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: role and per-wave constants stay off the vector unit
    const bool producer = wave >= kC3Consumers;
    const int cw = producer ? wave - kC3Consumers : wave;  // index inside the role
    const int wm = cw / WAVES_N, wn = cw % WAVES_N;
    const int ptid = tid - kC3Consumers * 64;   // producers: 0 .. NP*64-1

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
    const int halo_hw = p.HTH * p.HTW;
    const int ntaps = p.ntaps;
    const int nchunks = p.C_out / KC;
    const int nstages = ntaps * nchunks;

    SDGP_LDS int* rowpix = (SDGP_LDS int*)(smem + L::off_rowpix());
    SDGP_LDS unsigned char* lds_w = smem + L::off_w();
    SDGP_LDS unsigned char* lds_a = smem + L::off_a_h(p.nhalo);
    SDGP_LDS unsigned char* lds_meta = smem + L::off_meta(p.nhalo);
    SDGP_LDS unsigned char* lds_raw = smem + L::off_raw_h(p.nhalo);
    const int a_buf_bytes = L::a_bytes(p.nhalo), meta_buf_bytes = L::meta_bytes(p.nhalo);

    if (tid < kTileRows) {
        const int m = tid;
        int pix = -1;
        if (m < tile_rows) {
            const int tb = m / tile_hw, rem = m % tile_hw;
            const int th = rem / p.TW, tw = rem % p.TW;
            const int b = b0 + tb, hh = hh0 + th, ww = ww0 + tw;
            if (b < p.B && hh < p.H && ww < p.Wd) pix = (b * p.H + hh) * p.Wd + ww;
        }
        rowpix[m] = pix;
    }

    // gradient pixel (flat index into [B,P,Q]) of halo position hp, clamped into the tensor; ok = inside
    auto halo_pixel = [&](int hp, bool& ok) {
        const int tb = hp / halo_hw, rem = hp % halo_hw;
        const int hy = rem / p.HTW, hx = rem % p.HTW;
        const int b = b0 + tb, pp = hh0 + hy + p.dpmin, qq = ww0 + hx + p.dqmin;
        ok = hp < p.nhalo && b < p.B && pp >= 0 && pp < p.P && qq >= 0 && qq < p.Q;
        return ok ? (b * p.P + pp) * p.Q + qq : 0;
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int u = 0; u < TN; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.0f;

    // Number of whole-batch rounds that bring the first chunk's halo in (both roles count the same barriers).
    const int rounds0 = (p.nunits + kC3UnitsPerStep - 1) / kC3UnitsPerStep;

    if (producer) {
        // =============================================================== producers
        const int pw = cw;
        __builtin_amdgcn_s_setprio(3);  // few, short instructions: let them through ahead of the matrix waves
        // Loop-invariant values live in registers: nothing below reads the kernel arguments again.
        const uint16_t* const gW = p.W;
        const uint16_t* const gdO = p.dO;
        const int c_out = p.C_out, w_row = p.w_row, nunits = p.nunits, nhalo = p.nhalo;
        int my_woff = 0;                       // lane ti holds the W offset of tap ti (fetched with readlane)
        if (lane < ntaps) my_woff = p.taps[lane].woff;
        // per-lane W column (swizzled chunk) and row of each copy unit this wavefront owns
        uint32_t w_lane_off[WPW];  // bytes
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int uu = pw * WPW + i;
            const int row = uu * RPU + lane / CPR;
            const int lchunk = (lane % CPR) ^ (WSW * (row & 3));
            int col = n0 + lchunk * 8;
            if (col > p.C_in - 8) col = p.C_in - 8;  // columns past C_in feed accumulators that are never stored
            w_lane_off[i] = (uint32_t)(row * w_row + col) * 2u;
        }
        // halo position -> flat gradient pixel (clamped into the tensor), kept in LDS for the whole kernel
        // halo position -> address of channel 0 of its gradient pixel (the row of zeros when outside the image)
        typedef unsigned long long u64_t;
        SDGP_LDS u64_t* haloaddr = (SDGP_LDS u64_t*)(smem + L::off_halopix(p.nhalo));
        for (int hp = ptid; hp < L::pad8(nhalo); hp += NP * 64) {
            bool ok;
            const int gp = halo_pixel(hp, ok);
            haloaddr[hp] = ok ? (u64_t)(uintptr_t)(gdO + (size_t)gp * c_out) : (u64_t)(uintptr_t)kZeroRow;
        }
        const uint32_t c16_dense[2] = {(uint32_t)(((lane & 7) ^ ((lane >> 4) & 7)) * 16),
                                       (uint32_t)(((lane & 7) ^ ((4 + (lane >> 4)) & 7)) * 16)};
        const uint32_t c16_raw = (uint32_t)(((lane & 7) ^ (lane >> 3)) * 16);

        // W: the slab of stage (chunk, ti) into ring slot `slot`
        auto copy_w = [&](int chunk, int ti, int slot) {
            const int woff = __builtin_amdgcn_readlane(my_woff, ti);
            const uint16_t* src = gW + (size_t)chunk * KC * w_row + woff;
            const uint32_t dst = smem_base + L::off_w() + (uint32_t)slot * L::kWSlab + pw * WPW * 1024;
#pragma unroll
            for (int i = 0; i < WPW; ++i) copy16_to_lds(src, w_lane_off[i], dst + i * 1024);
        };
        // halo: copy unit u (8 pixels x 128 B of `chunk`) to LDS address dst (+ lane*16)
        auto copy_halo_unit = [&](int u, int chunk, uint32_t dst, bool dense_swizzle) {
            const u64_t a = haloaddr[u * 8 + (lane >> 3)];
            // the dense layout swizzles with (hp >> 1) & 7 = (4 * (u & 1) + (lane >> 4)) & 7
            const uint32_t c16 = dense_swizzle ? ((u & 1) ? c16_dense[1] : c16_dense[0]) : c16_raw;
            copy16_to_lds(reinterpret_cast<const void*>((uintptr_t)(a + (u64_t)(c16 + (uint32_t)chunk * (KC * 2)))), dst);
        };
        auto copy_sink = [&]() { copy16_to_lds(gW + lane * 8, smem_base + L::off_sink()); };

        // prune one raw batch (already in LDS slot `rslot`) into the compressed halo buffer of `chunk`
        // (a wavefront handles two units = 16 pixels; `rot` moves the busy wavefronts round the SIMDs)
        auto prune_batch = [&](int batch, int chunk, int rslot, int units_per_batch, int rot) {
            if constexpr (MODE != 0) {
                const int unit = 2 * ((pw + rot) & (NP - 1)) + ((lane >> 5) & 1), px = (ptid >> 2) & 7, part = ptid & 3;
                const int u = batch * units_per_batch + unit;
                const int hp = u * 8 + px;
                if (unit < units_per_batch && u < nunits && hp < nhalo) {
                    // flat element index of the pixel (an outside pixel is all zeros: any index gives zeros)
                    const uint64_t pix_e = (uint64_t)(haloaddr[hp] - (u64_t)(uintptr_t)gdO) >> 1;
                    SDGP_LDS unsigned char* src = lds_raw + rslot * L::kRawSlot + unit * 1024 + px * 128;
                    u32x4_t v[2];
                    v[0] = *(SDGP_LDS u32x4_t*)(src + (((2 * part) ^ px) * 16));
                    v[1] = *(SDGP_LDS u32x4_t*)(src + (((2 * part + 1) ^ px) * 16));
                    const uint64_t e0 = pix_e + (uint64_t)(chunk * KC + part * 16);
                    halo_item_to_lds<KC, MODE, M, RK, 16>(v, hp, part, e0, p.n, p.mix, lds_a + (chunk & 1) * a_buf_bytes,
                                                          lds_meta + (chunk & 1) * meta_buf_bytes);
                }
            }
        };
        __syncthreads();  // haloaddr visible to all producers (the consumers join this barrier too)

        // ---- prologue: first chunk's halo brought in synchronously
        if constexpr (MODE == 0) {
            for (int u = pw; u < nunits; u += NP) copy_halo_unit(u, 0, smem_base + L::off_a_h(p.nhalo) + u * 1024, true);
            wait_copies<0>();
            __syncthreads();
        } else {
            for (int r = 0; r < rounds0; ++r) {
#pragma unroll
                for (int j = 0; j < HPW; ++j) {
                    const int u = r * kC3UnitsPerStep + pw * HPW + j;
                    copy_halo_unit(u < nunits ? u : 0, 0, smem_base + L::off_raw_h(p.nhalo) + (pw * HPW + j) * 1024, false);
                }
                wait_copies<0>();
                __syncthreads();
                prune_batch(r, 0, 0, kC3UnitsPerStep, 0);
                __syncthreads();
            }
        }
        // Steady-state schedule.  "Issuing for stage g" requests the W slab of stage g+3 and the halo work tied to
        // stage g+3 (sparse: the raw batch that is pruned during stage g+3; dense: the units of window stage g).
        // (wc, wt) = (chunk, tap) of stage g+3; (gc, gt) = (chunk, tap) of stage g.  Both advance by one per issue.
        const int nb = SPARSE ? ntaps - 1 : ntaps - 3;  // stages of a chunk that carry halo work
        const int upb = (nunits + nb - 1) / nb;          // units per batch (<= 8, host-checked)
        int wc = 0, wt = 0, wslot = 0;                   // stage g+3, starting at stage 0 for g = -3
        int gc = 0, gt = 0;                              // stage g, valid once g >= 0
        auto issue = [&](bool g_valid) {
            // stages past the end re-copy the last slab into a slot nobody reads: the copy count stays exact
            const bool w_live = wc < nchunks;
            copy_w(w_live ? wc : nchunks - 1, w_live ? wt : ntaps - 1, wslot);
#pragma unroll
            for (int j = 0; j < HPW; ++j) {
                const int unit = pw * HPW + j;
                bool real = false;
                if constexpr (SPARSE) {
                    const int u = wt * upb + unit;       // batch wt of chunk wc+1 is pruned during stage (wc, wt)
                    real = w_live && wt < nb && wc + 1 < nchunks && unit < upb && u < nunits;
                    if (real) copy_halo_unit(u, wc + 1, smem_base + L::off_raw_h(p.nhalo) + wslot * L::kRawSlot + unit * 1024, false);
                } else {
                    const int u = gt * kC3UnitsPerStep + unit;  // dense: straight into the next chunk's buffer
                    real = g_valid && gc < nchunks && gt < nb && gc + 1 < nchunks && u < nunits;
                    if (real) copy_halo_unit(u, gc + 1, smem_base + L::off_a_h(p.nhalo) + ((gc + 1) & 1) * a_buf_bytes + u * 1024, true);
                }
                if (!real) copy_sink();
            }
            if (++wt == ntaps) wt = 0, ++wc;
            wslot = (wslot + 1) & (kC3Slots - 1);
            if (g_valid && ++gt == ntaps) gt = 0, ++gc;
        };
        static_assert(kC3Slots == kC3RawSlots, "the W ring and the raw halo ring advance together");
        issue(false);
        issue(false);
        issue(false);
        wait_copies<0>();
        __syncthreads();

        for (int g = 0; g < nstages; ++g) {
            const int pc = gc, pt = gt;  // (chunk, tap) of stage g, before issue() advances them
            issue(true);
            if constexpr (SPARSE) {
                if (pt < nb && pc + 1 < nchunks) prune_batch(pt, pc + 1, g & (kC3RawSlots - 1), upb, g);
            }
            // Only this stage's requests may still be in flight: the consumers read the fragments of stage g+1
            // before the barrier that ends stage g, so its slab (requested at stage g-2) must be complete one
            // barrier early.
            wait_copies<kPer>();
            __syncthreads();
        }
    } else {
        // =============================================================== consumers
        // per-lane row data: halo position and the set of taps that fall inside the image
        int rowbase[TM];  // halo position of each of this lane's rows (tap offsets are added per stage)
#pragma unroll
        for (int t = 0; t < TM; ++t) {
            const int m = wm * WM + t * 32 + (lane & 31);
            rowbase[t] = 0;
            if (m < tile_rows) {
                const int tb = m / tile_hw, rem = m % tile_hw;
                rowbase[t] = (tb * p.HTH + rem / p.TW) * p.HTW + rem % p.TW;
            }
        }
        int my_tap_off = 0;
        if (lane < ntaps) my_tap_off = (p.taps[lane].dp - p.dpmin) * p.HTW + (p.taps[lane].dq - p.dqmin);

        // B fragments: transpose reads from the swizzled slab, one lane address per 32-column tile
        int b_lane[TN];
#pragma unroll
        for (int u = 0; u < TN; ++u) {
            const int L16 = lane & 15;
            const int chunk = 8 * wn + 4 * u + 2 * ((lane >> 4) & 1) + ((L16 & 3) >> 1);
            b_lane[u] = (8 * (lane >> 5) + (L16 >> 2)) * L::kWRow + ((chunk ^ (WSW * (L16 >> 2))) * 16) + (L16 & 1) * 8;
        }

        __syncthreads();  // producers' halo table
        if constexpr (MODE == 0) {
            __syncthreads();
        } else {
            for (int r = 0; r < rounds0; ++r) {
                __syncthreads();
                __syncthreads();
            }
        }
        __syncthreads();  // end of the producers' prologue

        struct Frags {
            u32x4_t a[TM];
            int meta[TM];
            typename std::conditional<SPARSE, bf16x16_t, bf16x8_t>::type b[TN];
        };
        auto load_frags = [&](Frags& f, int slot, int chunk, int ti, int ks) {
            const int tap_off = __builtin_amdgcn_readlane(my_tap_off, ti);
            SDGP_LDS unsigned char* wbuf = lds_w + slot * L::kWSlab;
            SDGP_LDS unsigned char* abuf = lds_a + (chunk & 1) * a_buf_bytes;
#pragma unroll
            for (int t = 0; t < TM; ++t) {
                const int hp = rowbase[t] + tap_off;
                u32x4_t araw;
                if constexpr (SPARSE) {
                    araw = *(SDGP_LDS u32x4_t*)(abuf + hp * L::kAPitch + (lane >> 5) * 16 + ks * 32);
                    f.meta[t] = *(SDGP_LDS uint16_t*)(lds_meta + (chunk & 1) * meta_buf_bytes + hp * L::kMetaPitch +
                                                      (lane >> 5) * 2 + ks * 4);
                } else {
                    const int c16 = (ks * 2 + (lane >> 5)) ^ ((hp >> 1) & 7);
                    araw = *(SDGP_LDS u32x4_t*)(abuf + hp * 128 + c16 * 16);
                }
                f.a[t] = araw;
            }
            if constexpr (SPARSE) {
#pragma unroll
                for (int u = 0; u < TN; ++u) {
                    s16x4_t q[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (SDGP_LDS s16x4_t*)(wbuf + b_lane[u] + (ks * 32 + (i >> 1) * 16 + (i & 1) * 4) * L::kWRow));
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
                            (SDGP_LDS s16x4_t*)(wbuf + b_lane[u] + (ks * 16 + i * 4) * L::kWRow));
                    typedef short s16x8_t __attribute__((ext_vector_type(8)));
                    const s16x8_t all = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3]};
                    f.b[u] = __builtin_bit_cast(bf16x8_t, all);
                }
            }
        };
        auto mma = [&](const Frags& f) {
            bf16x8_t a[TM];
#pragma unroll
            for (int t = 0; t < TM; ++t) a[t] = __builtin_bit_cast(bf16x8_t, f.a[t]);
#pragma unroll
            for (int t = 0; t < TM; ++t)
#pragma unroll
                for (int u = 0; u < TN; ++u) {
                    if constexpr (SPARSE)
                        acc[t][u] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[t], f.b[u], acc[t][u], f.meta[t], 0, 0);
                    else
                        acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], f.b[u], acc[t][u], 0, 0, 0);
                }
        };

        // Fragments of k-step q+1 are requested before the matrix instructions of k-step q issue.  The next
        // stage's slab and halo are always complete one stage early (see the producers' schedule).
        static_assert(NKS % 2 == 0, "fragment double buffering alternates per k-step");
        Frags fr[2];
        int chunk = 0, ti = 0;
        load_frags(fr[0], 0, 0, 0, 0);
        for (int s = 0; s < nstages; ++s) {
            int nti = ti + 1, nchunk = chunk;
            if (nti == ntaps) nti = 0, ++nchunk;
            const int slot = s & (kC3Slots - 1), nslot = (s + 1) & (kC3Slots - 1);
            const bool has_next = s + 1 < nstages;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                // keep the order "request the next fragments, then issue this k-step's matrix instructions":
                // the reads then have a whole k-step of matrix work to land behind
                if (ks + 1 < NKS) load_frags(fr[(ks + 1) & 1], slot, chunk, ti, ks + 1);
                else if (has_next) load_frags(fr[0], nslot, nchunk, nti, 0);
#ifdef SDGP_C3_INTERLEAVE
                mma(fr[ks & 1]);
                // one matrix instruction, then a share of the next fragments' address arithmetic and LDS reads
#pragma unroll
                for (int i = 0; i < TM * TN; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, SDGP_C3_INTERLEAVE, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, SPARSE ? 2 : 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
#else
                __builtin_amdgcn_sched_barrier(0);
                mma(fr[ks & 1]);
                __builtin_amdgcn_sched_barrier(0);
#endif
            }
            __syncthreads();
            ti = nti, chunk = nchunk;
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
