// Backward-data kernel for stride-1 filters with 4..32 taps (3x3, 5x5): the layers where the product is bound by the
// matrix cores.  dL/dD = prune(dL/dO) (*) W as an implicit GEMM (Fig. 3 left; Sec. II-A): rows = input pixels,
// columns = input channels, reduction = taps x output channels, the pruned axis (Fig. 1).
//
// Design, from measurements on gfx950:
//   * Eight wavefronts, all of one kind: each owns a 128 x 64 (BN = 128) or 64 x 64 (BN = 64) register tile of a
//     512-row x BN-column workgroup tile and issues its share of the copies itself.  Two matrix wavefronts per SIMD
//     keep the matrix pipe fed while the other one waits for LDS; tiles of this size keep the LDS read traffic
//     (about 96 KB per 1024 matrix cycles) below what the LDS delivers.  Dedicated copy wavefronts would cost the
//     registers that such tiles need.
//   * Every byte from global memory moves with direct-to-LDS loads (lane i of a wavefront writes 16 bytes at LDS
//     base + 16 i).  They need no registers; a wavefront issues exactly two per stage and waits with a counter.
//   * The reduction runs in chunks of 32 channels.  One stage = (chunk, tap); one barrier per stage.  W slabs
//     (32 x BN, the layout W has in memory, 16-byte columns XOR-swizzled on the address side for the transpose
//     reads) go through a ring of 5 slots requested four stages ahead; a request is complete two stages after it
//     was issued, so fragments of stage s+1 can be read before the barrier that ends stage s.
//   * The gradient halo of a tile (the pixels its taps reach, clipped to the image) is brought in ONCE per chunk and
//     shared by all taps.  Dense: copied straight into the other halo buffer while the current chunk is multiplied.
//     Pruning (Sec. III-B): the raw halo streams through a ring of 4 batches; three stages after a batch was
//     requested the wavefronts rank / prune / compress it into the next chunk's halo buffer, two values and two
//     2-bit positions per aligned quad of channels -- the operand of v_smfmac_f32_32x32x32_bf16.  A gradient
//     element is ranked once per tile and chunk, not once per tap.
//   * Taps that fall outside the image read a row of zeros in LDS (one select per fragment address); nothing is
//     stored or copied for the padding.
//   * The result leaves through LDS: fp32 -> bf16, then 16-byte stores of whole pixel rows.
//
// Operand layouts of the matrix instructions and of ds_read_b64_tr_b16: see bwd_tiled.h.
#pragma once

#include <type_traits>

#include "bwd_tiled.h"

namespace sdgp {

struct WideParams {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    int B, P, Q, C_out, C_in, H, Wd;
    int R, S, pad, ntaps;
    int w_row;                   // elements per W row: R*S*C_in
    int n;
    uint32_t mix;
    int TB, TH, TW;              // tile: TB images x TH x TW pixels (<= 512)
    int tiles_h, tiles_w;
    int halo_max;                // upper bound of the halo pixels of any tile (LDS sizing)
    int hub;                     // pruning: copy units per raw batch
    int ntiles_n, nblocks;
};

constexpr int kWideRows = 512;
constexpr int kWideKC = 32;        // reduction channels per chunk
constexpr int kWideSlots = 5;      // W ring
constexpr int kWideAhead = 4;      // a slab is requested this many stages before its stage
constexpr int kWideRawSlots = 4;   // raw halo ring (pruning)
constexpr int kWideRawAhead = 3;
constexpr int kWideMaxTaps = 32;

template <int BN, int MODE>
struct WideLayout {
    static constexpr bool kSparse = MODE == 2;
    static constexpr int kWRow = BN * 2;
    static constexpr int kWSlab = kWideKC * kWRow;
    static constexpr int kWUnits = kWSlab / 1024;             // 1 KB copy units per slab (8 or 4)
    static constexpr int kHU = 16 - kWUnits;                   // halo copy units per stage (every wavefront issues two copies)
    static constexpr int kAPitch = kSparse ? 32 : 64;          // bytes per halo pixel in LDS
    static constexpr int kRawSlot = kHU * 1024;
    static constexpr int kOutPitch = BN * 2 + 16;
    __host__ __device__ static int pad16(int halo) { return (halo + 15) & ~15; }
    __host__ __device__ static int off_rowpix() { return 0; }   // survives the epilogue: the result tile starts after it
    __host__ __device__ static int off_out() { return kWideRows * 4; }
    __host__ __device__ static int off_w() { return off_out(); }
    __host__ __device__ static int off_sink() { return off_w() + kWideSlots * kWSlab; }
    __host__ __device__ static int off_zero() { return off_sink() + 1024; }
    __host__ __device__ static int off_haloaddr() { return off_zero() + 128; }
    __host__ __device__ static int off_raw(int halo) { return off_haloaddr() + pad16(halo) * 8; }
    __host__ __device__ static int off_a(int halo) { return off_raw(halo) + (kSparse ? kWideRawSlots * kRawSlot : 0); }
    __host__ __device__ static int a_bytes(int halo) { return pad16(halo) * kAPitch; }
    __host__ __device__ static int off_meta(int halo) { return off_a(halo) + 2 * a_bytes(halo); }
    __host__ __device__ static int meta_bytes(int halo) { return kSparse ? pad16(halo) * 4 : 0; }
    __host__ __device__ static int total(int halo) {
        const int loop = off_meta(halo) + 2 * meta_bytes(halo);
        const int out = off_out() + kWideRows * kOutPitch;  // the result tile is staged here after the last stage
        return loop > out ? loop : out;
    }
};

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_base + 16*i.  The compiler does not see
// these as memory instructions; callers count copies and wait with wide_wait_copies.
__device__ __forceinline__ void wide_copy16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
// Same, address = wave-uniform base + 32-bit byte offset per lane.
__device__ __forceinline__ void wide_copy16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}
// Waits until at most N of this wavefront's vector-memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wide_wait_copies() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Sixteen consecutive channels of one gradient pixel -> the compressed operand (Sec. III-B).
template <int M, int RK>
__device__ __forceinline__ void wide_prune16(const u32x4_t (&v)[2], int n, uint32_t mix, uint64_t e0, uint32_t (&packed)[4],
                                             uint32_t& meta) {
    if constexpr (RK != kRandom) {
        const uint32_t w[8] = {v[0][0], v[0][1], v[0][2], v[0][3], v[1][0], v[1][1], v[1][2], v[1][3]};
        prune_compress16_bf16<M, RK>(w, n, packed, meta);
    } else {
        uint32_t raw[16], out[16];
        bool keep[16];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                raw[i * 8 + 2 * x] = v[i][x] & 0xFFFFu;
                raw[i * 8 + 2 * x + 1] = v[i][x] >> 16;
            }
#pragma unroll
        for (int g = 0; g < 16 / M; ++g) {
            uint32_t r[M], o[M];
            bool kk[M];
#pragma unroll
            for (int j = 0; j < M; ++j) r[j] = raw[g * M + j];
            const uint64_t eg = e0 + (uint64_t)(g * M);
            prune_group<kBF16, M, RK, true>(r, n, hash_row(mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
            for (int j = 0; j < M; ++j) out[g * M + j] = o[j], keep[g * M + j] = kk[j];
        }
        meta = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool kq[4] = {keep[4 * q], keep[4 * q + 1], keep[4 * q + 2], keep[4 * q + 3]};
            const uint32_t oq[4] = {out[4 * q], out[4 * q + 1], out[4 * q + 2], out[4 * q + 3]};
            uint32_t v0, v1, pos;
            compress_quad(kq, oq, v0, v1, pos);
            packed[q] = v0 | (v1 << 16);
            meta |= pos << (4 * q);
        }
    }
}

template <int BN, int MODE, int M, int RK>
__global__ void __launch_bounds__(512) bwd_wide(const WideParams p) {
    using L = WideLayout<BN, MODE>;
    constexpr bool SPARSE = MODE == 2;
    constexpr int KC = kWideKC;
    constexpr int WAVES_N = BN / 64;
    constexpr int WAVES_M = 8 / WAVES_N;
    constexpr int WM = kWideRows / WAVES_M;
    constexpr int TM = WM / 32;
    constexpr int TN = 2;
    constexpr int KSTEP = SPARSE ? 32 : 16;
    constexpr int NKS = KC / KSTEP;
    constexpr int CPR = BN / 8;                 // 16-byte columns per W row
    constexpr int RPU = 1024 / L::kWRow;        // W rows per copy unit
    constexpr int WU = L::kWUnits;
    constexpr int HU = L::kHU;

    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDS unsigned char* smem = (SDGP_LDS unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar, so per-wave decisions stay off the vector unit
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
    // halo: the gradient pixels the tile's taps reach, clipped to the image (tap (r, s) reads pixel (h + pad - r, w + pad - s))
    const int py0 = max(0, hh0 + p.pad - (p.R - 1)), py1 = min(p.P, hh0 + p.TH + p.pad);
    const int qx0 = max(0, ww0 + p.pad - (p.S - 1)), qx1 = min(p.Q, ww0 + p.TW + p.pad);
    const int HTH = py1 - py0, HTW = qx1 - qx0;
    const int halo_hw = HTH * HTW;
    const int nhalo = p.TB * halo_hw;
    const int nunits = (nhalo + 15) >> 4;
    const int ntaps = p.ntaps;
    const int nchunks = p.C_out / KC;
    const int nstages = ntaps * nchunks;
    // Every workgroup walks the chunks and the taps in its own rotation.  The sum does not care, and the W slab of a
    // (chunk, tap) is then wanted by a few workgroups at a time instead of by all of them at once: all compute units
    // reading the same 8 KB in the same microsecond queue up at the few L2 channels that hold it.
    const int c_rot = mtile % nchunks, t_rot = (mtile / nchunks) % ntaps;
    auto phys_chunk = [&](int c) { const int x = c + c_rot; return x >= nchunks ? x - nchunks : x; };
    auto phys_tap = [&](int t) { const int x = t + t_rot; return x >= ntaps ? x - ntaps : x; };

    SDGP_LDS int* rowpix = (SDGP_LDS int*)(smem + L::off_rowpix());
    typedef unsigned long long u64_t;
    SDGP_LDS u64_t* haloaddr = (SDGP_LDS u64_t*)(smem + L::off_haloaddr());
    const uint32_t off_a = (uint32_t)L::off_a(p.halo_max), a_buf_bytes = (uint32_t)L::a_bytes(p.halo_max);
    const uint32_t off_meta = (uint32_t)L::off_meta(p.halo_max), meta_buf_bytes = (uint32_t)L::meta_bytes(p.halo_max);
    const uint32_t off_raw = (uint32_t)L::off_raw(p.halo_max);
    const uint16_t* const gdO = p.dO;
    const uint16_t* const gW = p.W;

    // ---- tables: output pixel of every tile row, address of channel 0 of every halo pixel, the row of zeros
    {
        const int m = tid;
        int pix = -1;
        if (m < tile_rows) {
            const int tb = m / tile_hw, rem = m % tile_hw;
            const int b = b0 + tb, hh = hh0 + rem / p.TW, ww = ww0 + rem % p.TW;
            if (b < p.B && hh < p.H && ww < p.Wd) pix = (b * p.H + hh) * p.Wd + ww;
        }
        rowpix[m] = pix;
    }
    for (int hp = tid; hp < L::pad16(nhalo); hp += 512) {
        size_t gp = 0;  // positions past the halo (tail of the last copy unit) copy pixel 0; nobody reads them
        if (hp < nhalo) {
            const int tb = hp / halo_hw, rem = hp % halo_hw;
            const int b = min(b0 + tb, p.B - 1);  // images past the batch: valid memory, rows never stored
            gp = ((size_t)b * p.P + (py0 + rem / HTW)) * p.Q + (qx0 + rem % HTW);
        }
        haloaddr[hp] = (u64_t)(uintptr_t)(gdO + gp * p.C_out);
    }
    if (tid < 32) {
        // 64 bytes of zero values; for the compressed format, positions (0, 1) in every quad at byte 64
        uint32_t z = 0;
        if (tid == 16) z = 0x44444444u;
        *(SDGP_LDS uint32_t*)(smem + L::off_zero() + tid * 4) = z;
    }

    // ---- per-lane row data: halo position of each row and the taps that fall inside the image
    int rowbase[TM];
    uint32_t tapmask[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        const int m = wm * WM + t * 32 + (lane & 31);
        rowbase[t] = 0, tapmask[t] = 0;
        if (m < tile_rows) {
            const int tb = m / tile_hw, rem = m % tile_hw;
            const int h = hh0 + rem / p.TW, w = ww0 + rem % p.TW;
            if (b0 + tb < p.B && h < p.H && w < p.Wd) {
                rowbase[t] = (tb * HTH + (h - py0)) * HTW + (w - qx0);
                uint32_t mask = 0;
                for (int r = 0; r < p.R; ++r)
                    for (int s = 0; s < p.S; ++s) {
                        const int pp = h + p.pad - r, qq = w + p.pad - s;
                        if (pp >= 0 && pp < p.P && qq >= 0 && qq < p.Q) mask |= 1u << (r * p.S + s);
                    }
                tapmask[t] = mask;
            }
        }
    }
    int my_tap_off = 0;  // lane ti holds the halo offset of tap ti (fetched with readlane)
    if (lane < ntaps) my_tap_off = (p.pad - lane / p.S) * HTW + (p.pad - lane % p.S);

    // ---- copy duties of this wavefront: two copies per stage
    // copy 0: a W unit (wavefronts below WU) or a halo unit; copy 1: a halo unit
    const bool w_duty = wave < WU;
    const int hj0 = wave - WU;                 // halo unit-in-stage of copy 0 (when not a W unit)
    const int hj1 = (8 - WU) + wave;           // halo unit-in-stage of copy 1
    uint32_t w_voff = 0;
    {
        const int row = (wave % WU) * RPU + lane / CPR;
        const int lchunk = (lane % CPR) ^ (2 * (row & 3));
        int col = n0 + lchunk * 8;
        if (col > p.C_in - 8) col = p.C_in - 8;  // columns past C_in feed accumulators that are never stored
        w_voff = (uint32_t)(row * p.w_row + col) * 2u;
    }
    // 16-byte column a lane copies: LDS position (lane & 3) of pixel (lane >> 2) holds the swizzled source column
    const uint32_t c16_halo = SPARSE ? (uint32_t)(((lane & 3) ^ ((lane >> 4) & 1)) * 16)
                                     : (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) * 16);

    auto copy_w = [&](int chunk, int ti, int slot) {  // logical (chunk, tap)
        const uint16_t* src = gW + ((size_t)phys_chunk(chunk) * KC * p.w_row + (size_t)phys_tap(ti) * p.C_in);
        wide_copy16(src, w_voff, smem_base + L::off_w() + (uint32_t)slot * L::kWSlab + (uint32_t)wave * 1024);
    };
    auto copy_halo = [&](int u, int chunk, uint32_t dst) {
        const u64_t a = haloaddr[u * 16 + (lane >> 2)];
        wide_copy16(reinterpret_cast<const void*>((uintptr_t)(a + (u64_t)(c16_halo + (uint32_t)phys_chunk(chunk) * (KC * 2)))), dst);
    };
    // keeps the copy count of a stage constant when there is no halo unit to bring: part of this workgroup's first slab
    auto copy_sink = [&]() {
        wide_copy16(gW + ((size_t)c_rot * KC * p.w_row + (size_t)t_rot * p.C_in), w_voff, smem_base + L::off_sink());
    };

    // rank / prune / compress one raw batch (in ring slot rslot) into the halo buffer of `chunk`
    auto prune_batch = [&](int batch, int chunk, int rslot, int units_per_batch, int rot) {
        if constexpr (SPARSE) {
            const int item = ((wave + rot) & 7) * 64 + lane;  // (unit, pixel, 16-channel half)
            const int j = item >> 5, px = (item >> 1) & 15, part = item & 1;
            const int u = batch * units_per_batch + j;
            const int hp = u * 16 + px;
            if (j < units_per_batch && hp < nhalo) {
                SDGP_LDS unsigned char* src = smem + off_raw + rslot * L::kRawSlot + j * 1024 + px * 64;
                const int sw = (px >> 2) & 1;
                u32x4_t v[2];
                v[0] = *(SDGP_LDS u32x4_t*)(src + (((2 * part) ^ sw) * 16));
                v[1] = *(SDGP_LDS u32x4_t*)(src + (((2 * part + 1) ^ sw) * 16));
                const uint64_t e0 = ((uint64_t)(haloaddr[hp] - (u64_t)(uintptr_t)gdO) >> 1) + (uint64_t)(phys_chunk(chunk) * KC + part * 16);
                uint32_t packed[4], meta;
                wide_prune16<M, RK>(v, p.n, p.mix, e0, packed, meta);
                const u32x4_t x = {packed[0], packed[1], packed[2], packed[3]};
                *(SDGP_LDS u32x4_t*)(smem + off_a + (chunk & 1) * a_buf_bytes + hp * 32 + ((part ^ ((hp >> 3) & 1)) * 16)) = x;
                *(SDGP_LDS uint16_t*)(smem + off_meta + (chunk & 1) * meta_buf_bytes + hp * 4 + part * 2) = (uint16_t)meta;
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

    __syncthreads();  // tables visible

    // ---- prologue: the first chunk's halo, the first W slabs, the first raw batches
    const int nb = SPARSE ? ntaps - 1 : ntaps - 3;  // stages of a chunk that carry halo work
    const int hub = SPARSE ? p.hub : HU;             // copy units per stage / batch
    if constexpr (!SPARSE) {
        for (int u = wave; u < nunits; u += 8) copy_halo(u, 0, smem_base + off_a + u * 1024);
    } else {
        const int rounds = (nunits + HU - 1) / HU;
        for (int r = 0; r < rounds; ++r) {
            for (int j = wave; j < HU; j += 8) {
                const int u = r * HU + j;
                if (u < nunits) copy_halo(u, 0, smem_base + off_raw + j * 1024);
            }
            wide_wait_copies<0>();
            __syncthreads();
            for (int rot = 0; rot < (HU * 32 + 511) / 512; ++rot) {
                // every wavefront takes 64 items per pass
                const int item = (rot * 8 + wave) * 64 + lane;
                const int j = item >> 5, px = (item >> 1) & 15, part = item & 1;
                const int hp = (r * HU + j) * 16 + px;
                if (j < HU && hp < nhalo) {
                    SDGP_LDS unsigned char* src = smem + off_raw + j * 1024 + px * 64;
                    const int sw = (px >> 2) & 1;
                    u32x4_t v[2];
                    v[0] = *(SDGP_LDS u32x4_t*)(src + (((2 * part) ^ sw) * 16));
                    v[1] = *(SDGP_LDS u32x4_t*)(src + (((2 * part + 1) ^ sw) * 16));
                    const uint64_t e0 = ((uint64_t)(haloaddr[hp] - (u64_t)(uintptr_t)gdO) >> 1) + (uint64_t)(c_rot * KC + part * 16);
                    uint32_t packed[4], meta;
                    wide_prune16<M, RK>(v, p.n, p.mix, e0, packed, meta);
                    const u32x4_t x = {packed[0], packed[1], packed[2], packed[3]};
                    *(SDGP_LDS u32x4_t*)(smem + off_a + hp * 32 + ((part ^ ((hp >> 3) & 1)) * 16)) = x;
                    *(SDGP_LDS uint16_t*)(smem + off_meta + hp * 4 + part * 2) = (uint16_t)meta;
                }
            }
            __syncthreads();
        }
    }

    // Stage bookkeeping (all scalar): (wc, wt) = (chunk, tap) of the stage whose W slab is requested next,
    // (rc, rt) = stage whose raw batch is requested next, (c, t) = current stage.
    int wc = 0, wt = 0, wslot = 0;
    int rc = 0, rt = 0, rslot = 0;
    auto issue_w = [&]() {
        if (w_duty) {
            const bool live = wc < nchunks;  // past the end: the last slab again, into a slot nobody reads
            copy_w(live ? wc : nchunks - 1, live ? wt : ntaps - 1, wslot);
        }
        if (++wt == ntaps) wt = 0, ++wc;
        if (++wslot == kWideSlots) wslot = 0;
    };
    // raw batch that is pruned during stage (rc, rt): batch rt of chunk rc + 1
    auto issue_raw = [&](int j) {
        const int u = rt * hub + j;
        const bool real = rc + 1 < nchunks && rt < nb && j < hub && u < nunits;
        if (real) copy_halo(u, rc + 1, smem_base + off_raw + rslot * L::kRawSlot + j * 1024);
        return real;
    };
    auto advance_raw = [&]() {
        if (++rt == ntaps) rt = 0, ++rc;
        rslot = (rslot + 1) & (kWideRawSlots - 1);
    };
    for (int i = 0; i < kWideAhead; ++i) issue_w();
    if constexpr (SPARSE) {
        for (int i = 0; i < kWideRawAhead; ++i) {
            if (!w_duty) issue_raw(hj0);
            issue_raw(hj1);
            advance_raw();
        }
    }
    wide_wait_copies<0>();
    __syncthreads();

    // ---- fragments
    uint32_t b_lane[TN];  // transpose reads from the swizzled slab, one lane address per 32-column tile
#pragma unroll
    for (int u = 0; u < TN; ++u) {
        const int L16 = lane & 15;
        const int chunk = 8 * wn + 4 * u + 2 * ((lane >> 4) & 1) + ((L16 & 3) >> 1);
        b_lane[u] = (uint32_t)((8 * (lane >> 5) + (L16 >> 2)) * L::kWRow + ((chunk ^ (2 * (L16 >> 2))) * 16) + (L16 & 1) * 8);
    }
    struct Frags {
        u32x4_t a[TM];
        int meta[TM];
        typename std::conditional<SPARSE, bf16x16_t, bf16x8_t>::type b[TN];
    };
    uint32_t a_addr[TM];   // LDS address of this lane's A fragment of the stage being loaded (k-step 0)
    uint32_t m_addr[TM];
    const uint32_t half = (uint32_t)(lane >> 5);
    // addresses for stage (chunk, ti)
    auto stage_addr = [&](int chunk, int ti) {
        const int pti = phys_tap(ti);
        const int tap_off = __builtin_amdgcn_readlane(my_tap_off, pti);
        const uint32_t abuf = off_a + (uint32_t)(chunk & 1) * a_buf_bytes;
#pragma unroll
        for (int t = 0; t < TM; ++t) {
            const uint32_t hp = (uint32_t)(rowbase[t] + tap_off);
            const bool inside = (tapmask[t] >> pti) & 1u;
            if constexpr (SPARSE) {
                const uint32_t a = abuf + hp * 32u + ((half ^ ((hp >> 3) & 1u)) << 4);
                const uint32_t mm = off_meta + (uint32_t)(chunk & 1) * meta_buf_bytes + hp * 4u + half * 2u;
                a_addr[t] = inside ? a : (uint32_t)L::off_zero();
                m_addr[t] = inside ? mm : (uint32_t)L::off_zero() + 64u;
            } else {
                const uint32_t a = abuf + hp * 64u + ((half ^ ((hp >> 2) & 3u)) << 4);
                a_addr[t] = inside ? a : (uint32_t)L::off_zero();
            }
        }
    };
    auto load_frags = [&](Frags& f, int slot, int ks) {
        SDGP_LDS unsigned char* wbuf = smem + L::off_w() + slot * L::kWSlab;
#pragma unroll
        for (int t = 0; t < TM; ++t) {
            if constexpr (SPARSE) {
                f.a[t] = *(SDGP_LDS u32x4_t*)(smem + a_addr[t]);
                f.meta[t] = *(SDGP_LDS uint16_t*)(smem + m_addr[t]);
            } else {
                f.a[t] = *(SDGP_LDS u32x4_t*)(smem + (a_addr[t] ^ (uint32_t)(ks * 32)));
            }
        }
#pragma unroll
        for (int u = 0; u < TN; ++u) {
            if constexpr (SPARSE) {
                s16x4_t q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (SDGP_LDS s16x4_t*)(wbuf + b_lane[u] + ((i >> 1) * 16 + (i & 1) * 4) * L::kWRow));
                typedef short s16x16_t __attribute__((ext_vector_type(16)));
                const s16x16_t all = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3],
                                      q[2][0], q[2][1], q[2][2], q[2][3], q[3][0], q[3][1], q[3][2], q[3][3]};
                f.b[u] = __builtin_bit_cast(bf16x16_t, all);
            } else {
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

    // ---- main loop.  Fragments of the next k-step are requested before the matrix instructions of the current
    // one; at a stage's last k-step that is the next stage, whose slab and halo are complete one barrier early.
    int c = 0, t = 0, slot = 0;       // current stage
    Frags fr[2];
    stage_addr(0, 0);
    load_frags(fr[0], 0, 0);
    // one k-step; CUR selects the fragment set (compile-time)
    auto kstep = [&](Frags& cur, Frags& nxt, int ks, int s) {
        if (ks == 0) {
            // this stage's copies: the W slab four stages ahead, and halo work
            issue_w();
            if constexpr (SPARSE) {
                bool r0 = w_duty, r1;
                if (!w_duty) r0 = issue_raw(hj0);
                r1 = issue_raw(hj1);
                advance_raw();
                if (!r0) copy_sink();
                if (!r1) copy_sink();
                if (t < nb && c + 1 < nchunks) prune_batch(t, c + 1, s & (kWideRawSlots - 1), hub, s);
            } else {
                // dense: units of the next chunk straight into the other halo buffer
                const bool on = t < nb && c + 1 < nchunks;
                const uint32_t dstb = smem_base + off_a + (uint32_t)((c + 1) & 1) * a_buf_bytes;
                bool r0 = w_duty, r1 = false;
                if (!w_duty) {
                    const int u = t * HU + hj0;
                    r0 = on && u < nunits;
                    if (r0) copy_halo(u, c + 1, dstb + u * 1024);
                }
                {
                    const int u = t * HU + hj1;
                    r1 = on && u < nunits;
                    if (r1) copy_halo(u, c + 1, dstb + u * 1024);
                }
                if (!r0) copy_sink();
                if (!r1) copy_sink();
            }
        }
        const bool last = ks == NKS - 1;
        if (!last) {
            load_frags(nxt, slot, ks + 1);
        } else if (s + 1 < nstages) {
            int nt = t + 1, nc = c;
            if (nt == ntaps) nt = 0, ++nc;
            stage_addr(nc, nt);
            load_frags(nxt, slot + 1 == kWideSlots ? 0 : slot + 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        mma(cur);
        __builtin_amdgcn_sched_barrier(0);
        if (last) {
            wide_wait_copies<4>();  // everything requested two stages ago has landed
            __syncthreads();
            if (++t == ntaps) t = 0, ++c;
            if (++slot == kWideSlots) slot = 0;
        }
    };
    if constexpr (NKS == 2) {
        for (int s = 0; s < nstages; ++s) {
            kstep(fr[0], fr[1], 0, s);
            kstep(fr[1], fr[0], 1, s);
        }
    } else {
        int s = 0;
        for (; s + 1 < nstages; s += 2) {
            kstep(fr[0], fr[1], 0, s);
            kstep(fr[1], fr[0], 0, s + 1);
        }
        if (s < nstages) kstep(fr[0], fr[1], 0, s);
    }

    // ---- epilogue: fp32 -> bf16 (RNE) into LDS, then whole pixel rows with 16-byte stores
    wide_wait_copies<0>();
    __syncthreads();  // nobody reads or copies into the loop's buffers any more
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    SDGP_LDS unsigned char* outb = smem + L::off_out();
#pragma unroll
    for (int tt = 0; tt < TM; ++tt)
#pragma unroll
        for (int u = 0; u < TN; ++u)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                // registers r and r + 1 are two consecutive rows of one column
                const int m = wm * WM + tt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int col = wn * 64 + u * 32 + (lane & 31);
                const f32x2_t v = {acc[tt][u][r], acc[tt][u][r + 1]};
                const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
                *(SDGP_LDS uint16_t*)(outb + m * L::kOutPitch + col * 2) = (uint16_t)pk;
                *(SDGP_LDS uint16_t*)(outb + (m + 1) * L::kOutPitch + col * 2) = (uint16_t)(pk >> 16);
            }
    __syncthreads();
#pragma unroll 4
    for (int idx = tid; idx < kWideRows * CPR; idx += 512) {
        const int m = idx / CPR, cc = idx % CPR;
        const int pix = rowpix[m];
        if (pix >= 0 && n0 + cc * 8 < p.C_in) {
            const u32x4_t v = *(SDGP_LDS u32x4_t*)(outb + m * L::kOutPitch + cc * 16);
            *reinterpret_cast<u32x4_t*>(p.dD + (size_t)pix * p.C_in + n0 + cc * 8) = v;
        }
    }
}

}  // namespace sdgp
