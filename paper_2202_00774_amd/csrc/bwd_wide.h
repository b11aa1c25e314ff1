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
//     Pruning (Sec. III-B, 3x3 filters): the raw halo of the next chunk streams into a ring of two 16 KB slots, a
//     third of the halo at a time; at taps 1, 4 and 7 all wavefronts together rank / prune / compress one third
//     (one 16-channel item per lane) into the next chunk's halo buffer, two values and two 2-bit positions per
//     aligned quad of channels -- the operand of v_smfmac_f32_32x32x32_bf16.  Whole-workgroup passes keep the
//     lanes full and the wavefronts level at the barrier; a gradient element is ranked once per tile and chunk,
//     not once per tap.
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
    int hub;                     // pruning: copy units per pass (a third of the halo, at most 16)
    int ntiles_n, nblocks;
    int exp;                     // development aid (builds with SDGP_TRACE only): switches parts of the kernel off
};

constexpr int kWideRows = 512;
constexpr int kWideKC = 32;        // reduction channels per chunk
constexpr int kWideSlots = 5;      // W ring
constexpr int kWideAhead = 4;      // a slab is requested this many stages before its stage
constexpr int kWideRawSlots = 2;   // raw halo ring (pruning): two passes of up to 16 copy units
constexpr int kWidePassUnits = 16; // 16 units = 256 pixels = 512 items of 16 channels: one item per lane of the workgroup
constexpr int kWidePasses = 3;     // pruning passes per chunk, at taps 1, 4 and 7 of a 9-tap filter
constexpr int kWideRawAhead = 4;   // the raw stream runs this many stages ahead of the current stage
constexpr int kWideMaxTaps = 9;      // the per-(tap, row) address table lives in LDS

template <int BN, int MODE>
struct WideLayout {
    static constexpr bool kSparse = MODE == 2;
    static constexpr int kWRow = BN * 2;
    static constexpr int kWSlab = kWideKC * kWRow;
    static constexpr int kWUnits = kWSlab / 1024;             // 1 KB copy units per slab (8 or 4)
    static constexpr int kHU = 16 - kWUnits;                   // halo copy units per stage (every wavefront issues two copies)
    static constexpr int kAPitch = kSparse ? 32 : 64;          // bytes per halo pixel in LDS
    static constexpr int kRawSlot = kWidePassUnits * 1024;
    static constexpr int kOutPitch = BN * 2 + 16;
    // halo pixels of a buffer: the copy units, then one all-zero pixel that taps outside the image read
    __host__ __device__ static int pad16(int halo) { return (halo + 15) & ~15; }
    __host__ __device__ static int pixels(int halo) { return pad16(halo) + 16; }
    __host__ __device__ static int zero_pixel(int halo) { return (halo + 15) & ~15; }
    __host__ __device__ static int off_rowpix() { return 0; }   // survives the epilogue: the result tile starts after it
    __host__ __device__ static int off_out() { return kWideRows * 4; }
    __host__ __device__ static int off_w() { return off_out(); }
    __host__ __device__ static int off_sink() { return off_w() + kWideSlots * kWSlab; }
    __host__ __device__ static int off_atab() { return off_sink() + 1024; }
    __host__ __device__ static int off_haloaddr() { return off_atab() + kWideMaxTaps * kWideRows * 4; }
    __host__ __device__ static int off_raw(int halo) { return off_haloaddr() + pixels(halo) * 8; }
    __host__ __device__ static int off_a(int halo) { return off_raw(halo) + (kSparse ? kWideRawSlots * kRawSlot : 0); }
    __host__ __device__ static int a_bytes(int halo) { return pixels(halo) * kAPitch; }
    __host__ __device__ static int off_meta(int halo) { return off_a(halo) + 2 * a_bytes(halo); }
    __host__ __device__ static int meta_bytes(int halo) { return kSparse ? pixels(halo) * 4 : 0; }
    __host__ __device__ static int total(int halo) {
        const int loop = off_meta(halo) + 2 * meta_bytes(halo);
        const int out = off_out() + kWideRows * kOutPitch;  // the result tile is staged here after the last stage
        return loop > out ? loop : out;
    }
};

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_base + 16*i.  The compiler does not see
// these as memory instructions; callers count copies and wait with wide_wait_copies.
__device__ __forceinline__ void wide_copy16(const void* gptr, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);  // wave-uniform by construction
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(gptr) : "memory");
}
// Same, address = wave-uniform base + 32-bit byte offset per lane.
__device__ __forceinline__ void wide_copy16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
    const uint64_t a = (uint64_t)(uintptr_t)sbase;
    // (the builtin returns a signed int: go through uint32_t, or the low word sign-extends into the high one)
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
    const uint64_t ua = ((uint64_t)hi << 32) | (uint64_t)lo;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(base), "v"(voff), "s"(ua) : "memory");
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

#ifdef SDGP_TRACE
#define SDGP_EXP(bit) (p.exp & (bit))
#else
#define SDGP_EXP(bit) false
#endif

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

    SDGP_LDS int* rowpix = (SDGP_LDS int*)(smem + L::off_rowpix());
    typedef unsigned long long u64_t;
    SDGP_LDS u64_t* haloaddr = (SDGP_LDS u64_t*)(smem + L::off_haloaddr());
    SDGP_LDS uint32_t* atab = (SDGP_LDS uint32_t*)(smem + L::off_atab());
    const uint32_t off_a = (uint32_t)L::off_a(p.halo_max), a_buf_bytes = (uint32_t)L::a_bytes(p.halo_max);
    const uint32_t off_meta = (uint32_t)L::off_meta(p.halo_max), meta_buf_bytes = (uint32_t)L::meta_bytes(p.halo_max);
    const uint32_t off_raw = (uint32_t)L::off_raw(p.halo_max);
    const uint32_t zero_pix = (uint32_t)L::zero_pixel(p.halo_max);
    const uint16_t* const gdO = p.dO;
    const uint16_t* const gW = p.W;

    // ---- tables (one row of the tile per thread)
    //   rowpix[m]        output pixel of tile row m (-1: none)
    //   atab[tap][m]     byte offset, inside a halo buffer, of the gradient pixel that physical tap `tap` of row m reads
    //                    (dense: with the pixel's swizzle; the zero pixel when the tap falls outside the image)
    //   haloaddr[hp]     address of channel 0 of halo pixel hp
    {
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
        for (int r = 0; r < p.R; ++r)
            for (int sx = 0; sx < p.S; ++sx) {
                const int pp = h + p.pad - r, qq = w + p.pad - sx;
                const bool inside = live && pp >= 0 && pp < p.P && qq >= 0 && qq < p.Q;
                const uint32_t hp = inside ? (uint32_t)(rowbase + (p.pad - r) * HTW + (p.pad - sx)) : zero_pix;
                atab[(r * p.S + sx) * kWideRows + m] = SPARSE ? hp * 32u : hp * 64u + (((hp >> 2) & 3u) << 4);
            }
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
    if (tid < 64) {
        // the zero pixel of both halo buffers; compressed format: values 0 and positions (0, 1) in every quad
        const uint32_t buf = tid >> 5, i = tid & 31;
        if (i < L::kAPitch / 4) *(SDGP_LDS uint32_t*)(smem + off_a + buf * a_buf_bytes + zero_pix * L::kAPitch + i * 4) = 0u;
        if (SPARSE && i == 31) *(SDGP_LDS uint32_t*)(smem + off_meta + buf * meta_buf_bytes + zero_pix * 4) = 0x44444444u;
    }

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
    const uint32_t haloaddr_lane = (uint32_t)L::off_haloaddr() + (uint32_t)(lane >> 2) * 8u;

    // unit u of the halo, channels at byte offset src_off of every pixel, to LDS address dst
    auto copy_halo = [&](int u, uint32_t src_off, uint32_t dst) {
        const u64_t a = *(SDGP_LDS u64_t*)(smem + haloaddr_lane + (uint32_t)u * 128u);
        wide_copy16(reinterpret_cast<const void*>((uintptr_t)(a + (u64_t)(c16_halo + src_off))), dst);
    };
    const uint32_t tapB = (uint32_t)p.C_in * 2u;                 // bytes between the slabs of consecutive taps
    const uint32_t chunkB = (uint32_t)KC * (uint32_t)p.w_row * 2u;  // ... of consecutive chunks
    const unsigned char* const gWb = reinterpret_cast<const unsigned char*>(gW);
    // keeps the copy count of a stage constant when there is no halo unit to bring: part of this workgroup's first slab
    auto copy_sink = [&]() {
        wide_copy16(gWb + ((size_t)c_rot * chunkB + (size_t)t_rot * tapB), w_voff, smem_base + L::off_sink());
    };

    // rank / prune / compress 64 items (pixel, 16-channel half) of a raw batch into a halo buffer (Sec. III-B)
    //   item0: first item of this wavefront; u0: first halo unit of the batch; raw: LDS offset of the batch
    auto prune_items = [&](int item0, int nitems, int u0, uint32_t raw, uint32_t abuf, uint32_t mbuf, uint32_t chan0) {
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
                wide_prune16<M, RK>(v, p.n, p.mix, e0, packed, meta);
                const u32x4_t x = {packed[0], packed[1], packed[2], packed[3]};
                *(SDGP_LDS u32x4_t*)(smem + abuf + hp * 32 + part * 16) = x;
                *(SDGP_LDS uint16_t*)(smem + mbuf + hp * 4 + part * 2) = (uint16_t)meta;
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

    // ---- prologue: the first chunk's halo (physical chunk c_rot)
    const int nb = SPARSE ? ntaps - 1 : ntaps - 3;  // stages of a chunk that carry halo work
    const int hub = SPARSE ? p.hub : HU;             // copy units per stage / batch
    if constexpr (!SPARSE) {
        for (int u = wave; u < nunits; u += 8) copy_halo(u, (uint32_t)c_rot * (KC * 2), smem_base + off_a + u * 1024);
    } else {
        const int rounds = (nunits + kWidePassUnits - 1) / kWidePassUnits;
        for (int r = 0; r < rounds; ++r) {
            for (int j = wave; j < kWidePassUnits; j += 8)
                if (r * kWidePassUnits + j < nunits)
                    copy_halo(r * kWidePassUnits + j, (uint32_t)c_rot * (KC * 2), smem_base + off_raw + j * 1024);
            wide_wait_copies<0>();
            __syncthreads();
            prune_items(wave * 64, kWidePassUnits * 32, r * kWidePassUnits, off_raw, off_a, off_meta, (uint32_t)c_rot * KC);
            __syncthreads();
        }
    }

    // ---- stage bookkeeping, all scalar and incremental.
    // W stream: the slab requested next (kWideAhead stages ahead of the current stage).  Past the last stage it
    // keeps walking valid slabs into slots nobody reads, so the copy count per stage stays constant.
    uint32_t w_tap_off = (uint32_t)t_rot * tapB, w_chunk_off = (uint32_t)c_rot * chunkB;
    const uint32_t w_tap_end = (uint32_t)ntaps * tapB, w_chunk_end = (uint32_t)nchunks * chunkB;
    int w_t = 0;
    uint32_t w_dst = smem_base + L::off_w() + (uint32_t)wave * 1024;
    const uint32_t w_dst_end = smem_base + L::off_w() + kWideSlots * L::kWSlab + (uint32_t)wave * 1024;
    auto issue_w = [&]() {
        if (w_duty && !SDGP_EXP(4)) wide_copy16(gWb + ((size_t)w_chunk_off + w_tap_off), w_voff, w_dst);
        w_tap_off += tapB;
        if (w_tap_off == w_tap_end) w_tap_off = 0;
        if (++w_t == ntaps) {
            w_t = 0;
            w_chunk_off += chunkB;
            if (w_chunk_off == w_chunk_end) w_chunk_off = 0;
        }
        w_dst += L::kWSlab;
        if (w_dst == w_dst_end) w_dst -= kWideSlots * L::kWSlab;
    };
    // halo stream.  Dense: units of the next chunk, requested during the current chunk's first nb stages, straight
    // into the other halo buffer.  Pruning: the raw stream runs kWideRawAhead stages ahead in a cycle of three steps
    // per pass -- first half of the pass's units, second half, nothing -- into ring slot (pass & 1).
    // h_u0 = first unit of the step, h_lim = one past the last unit to bring (0: none), h_pc = physical chunk.
    int h_t = 0, h_c = 0;                 // dense: stage the stream works for.  pruning: step in the cycle, pass in the chunk
    int h_u0 = 0;
    int h_pc = c_rot + 1 == nchunks ? 0 : c_rot + 1;  // physical chunk the stream fetches
    const int h_cap = nb * hub;
    int h_lim = nchunks > 1 ? min(nunits, SPARSE ? hub : h_cap) : 0;
    int h_chunk = 1;                       // pruning: logical chunk the stream fetches
    uint32_t h_raw = smem_base + off_raw;  // pruning: where unit h_u0 of the step lands
    uint32_t h_slot = 0;
    uint32_t h_buf = smem_base + off_a + a_buf_bytes;  // dense: the halo buffer being filled
    // The pixel addresses of the units a wavefront copies next are fetched from the table one stage early
    // (slot 0: unit-in-stage hj0, slot 1: hj1), so the copy itself never waits for LDS.
    u64_t h_addr[2] = {0, 0};
    auto halo_prefetch = [&]() {
        if (!w_duty && h_u0 + hj0 < h_lim) h_addr[0] = *(SDGP_LDS u64_t*)(smem + haloaddr_lane + (uint32_t)(h_u0 + hj0) * 128u);
        if (h_u0 + hj1 < h_lim) h_addr[1] = *(SDGP_LDS u64_t*)(smem + haloaddr_lane + (uint32_t)(h_u0 + hj1) * 128u);
    };
    auto halo_copy = [&](int slot) {  // returns whether a copy was issued
        const int j = slot ? hj1 : hj0;
        const int u = h_u0 + j;
        const bool real = u < h_lim && !SDGP_EXP(4);
        if (real)
            wide_copy16(reinterpret_cast<const void*>((uintptr_t)(h_addr[slot] + (u64_t)(c16_halo + (uint32_t)h_pc * (KC * 2)))),
                        SPARSE ? h_raw + (uint32_t)j * 1024u : h_buf + (uint32_t)u * 1024u);
        return real;
    };
    auto halo_advance = [&]() {
        if constexpr (SPARSE) {
            // h_t: step in the cycle (0, 1: halves of the pass; 2: idle), h_c: pass in the chunk
            ++h_t;
            if (h_t == 1) {
                h_u0 += HU, h_raw += HU * 1024;       // second half: the pass's remaining units
            } else if (h_t == 2) {
                h_lim = 0;                            // idle step
            } else {
                h_t = 0;
                h_slot ^= 1u;
                if (++h_c == kWidePasses) {
                    h_c = 0, ++h_chunk;
                    h_pc = h_pc + 1 == nchunks ? 0 : h_pc + 1;
                }
                h_u0 = h_c * hub;
                h_raw = smem_base + off_raw + h_slot * L::kRawSlot;
                h_lim = h_chunk < nchunks ? min(nunits, h_u0 + hub) : 0;
            }
        } else {
            h_u0 += hub;
            if (++h_t == ntaps) {
                h_t = 0, h_u0 = 0, ++h_c;
                h_pc = h_pc + 1 == nchunks ? 0 : h_pc + 1;
                h_lim = h_c + 1 < nchunks ? min(nunits, h_cap) : 0;
                h_buf = (h_c & 1) ? smem_base + off_a : smem_base + off_a + a_buf_bytes;
            }
        }
        halo_prefetch();
    };
    // the stage's copy 0 when it is not a W unit, and copy 1; a stand-in copy keeps the count per stage constant
    auto issue_halo0 = [&]() {
        if (!w_duty && !halo_copy(0) && !SDGP_EXP(4)) copy_sink();
    };
    auto issue_halo1 = [&]() {
        const bool r1 = halo_copy(1);
        halo_advance();
        if (!r1 && !SDGP_EXP(4)) copy_sink();
    };
    for (int i = 0; i < kWideAhead; ++i) issue_w();
    halo_prefetch();
    if constexpr (SPARSE) {
        for (int i = 0; i < kWideRawAhead; ++i) {
            if (!w_duty) halo_copy(0);
            halo_copy(1);
            halo_advance();
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
        b_lane[u] = (uint32_t)(L::off_w() + (8 * (lane >> 5) + (L16 >> 2)) * L::kWRow + ((chunk ^ (2 * (L16 >> 2))) * 16) +
                               (L16 & 1) * 8);
    }
    struct Frags {
        u32x4_t a[TM];
        int meta[TM];
        typename std::conditional<SPARSE, bf16x16_t, bf16x8_t>::type b[TN];
    };
    const uint32_t half = (uint32_t)(lane >> 5);
    const uint32_t atab_lane = (uint32_t)L::off_atab() + (uint32_t)(wm * WM + (lane & 31)) * 4u;
    uint32_t a_ent[TM];    // table entries of the stage whose fragments are being loaded
    uint32_t a_ent_n[TM];  // ... of the stage after it (requested a k-step early)
    auto read_entries = [&](int ptap) {
#pragma unroll
        for (int t = 0; t < TM; ++t) a_ent_n[t] = *(SDGP_LDS uint32_t*)(smem + atab_lane + (uint32_t)ptap * (kWideRows * 4) + t * 128);
    };
    // dense: a_lo = lane part of the address (half, k-step); pruning: value and position addresses
    const uint32_t a_k0 = SPARSE ? half * 16u : half << 4;
    const uint32_t m_k0 = half * 2u;
    // fragment requests, in pieces small enough to sit between two matrix instructions
    auto load_a = [&](Frags& f, int t, uint32_t abuf, uint32_t mbuf, int ks) {
        if (SDGP_EXP(8)) return;
        if constexpr (SPARSE) {
            f.a[t] = *(SDGP_LDS u32x4_t*)(smem + ((a_ent[t] | a_k0) + abuf));
            f.meta[t] = *(SDGP_LDS uint16_t*)(smem + (((a_ent[t] >> 3) | m_k0) + mbuf));
        } else {
            f.a[t] = *(SDGP_LDS u32x4_t*)(smem + ((a_ent[t] ^ (a_k0 | (uint32_t)(ks * 32))) + abuf));
        }
    };
    auto load_b = [&](Frags& f, int u, uint32_t wslot_off, int ks) {
        if (SDGP_EXP(8)) return;
        SDGP_LDS unsigned char* wb = smem + b_lane[u] + wslot_off;
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
    auto load_frags = [&](Frags& f, uint32_t abuf, uint32_t mbuf, uint32_t wslot_off, int ks) {
#pragma unroll
        for (int t = 0; t < TM; ++t) load_a(f, t, abuf, mbuf, ks);
#pragma unroll
        for (int u = 0; u < TN; ++u) load_b(f, u, wslot_off, ks);
    };
    auto mma_one = [&](const Frags& f, int t, int u) {
        if (SDGP_EXP(2)) return;
        const bf16x8_t a = __builtin_bit_cast(bf16x8_t, f.a[t]);
        if constexpr (SPARSE)
            acc[t][u] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, f.b[u], acc[t][u], f.meta[t], 0, 0);
        else
            acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, f.b[u], acc[t][u], 0, 0, 0);
    };

    // ---- main loop.  A matrix instruction occupies the pipe for 32 cycles; a wavefront issues in order, one
    // instruction every four to five cycles.  Everything else a stage needs -- the copies, their bookkeeping, the
    // requests for the next k-step's fragments -- is therefore cut into pieces of a few instructions and placed
    // BETWEEN the matrix instructions, where it costs nothing.  Fragments are requested one k-step ahead; at a
    // stage's last k-step that is the next stage, whose slab and halo are complete one barrier early.
    int t = 0, c = 0;                    // current stage: logical tap and chunk
    int ptap_next = t_rot + 1 == ntaps ? 0 : t_rot + 1;   // physical tap of the next stage
    int pc_next = c_rot + 1 == nchunks ? 0 : c_rot + 1;   // physical chunk of the next chunk
    uint32_t abuf = off_a, mbuf = off_meta;               // halo buffer of the current chunk
    uint32_t abuf_other = off_a + a_buf_bytes, mbuf_other = off_meta + meta_buf_bytes;
    uint32_t wslot_off = 0;                                // byte offset of the current stage's slab in the ring
    Frags fr[2];
    read_entries(t_rot);
#pragma unroll
    for (int i = 0; i < TM; ++i) a_ent[i] = a_ent_n[i];
    load_frags(fr[0], abuf, mbuf, 0, 0);
    constexpr int GAPS = TM * TN;        // matrix instructions of a k-step
    constexpr int APIECES = (TM + 1) / 2;
    auto kstep = [&](Frags& cur, Frags& nxt, int ks, int s) {
        const bool last = ks == NKS - 1;
        const bool more = s + 1 < nstages;
        const uint32_t wslot_next = wslot_off + L::kWSlab == kWideSlots * L::kWSlab ? 0u : wslot_off + L::kWSlab;
        const bool chunk_ends = t + 1 == ntaps;
        // where this k-step's fragment requests go: the next k-step of this stage, or the first one of the next stage
        const uint32_t la = (last && chunk_ends) ? abuf_other : abuf, lm = (last && chunk_ends) ? mbuf_other : mbuf;
        const uint32_t lw = last ? wslot_next : wslot_off;
        const int lks = last ? 0 : ks + 1;
        const bool do_load = !last || more;
        const bool copies = ks == 0;     // the stage's copies ride on its first k-step
        if (SPARSE && more) read_entries(ptap_next);
        // pieces, in issue order
        //   0            table entries: dense first k-step requests them, a last k-step takes them over
        //   1..APIECES   A fragments of two row tiles each
        //   then TN      B fragments of one column tile each
        //   then 3       the W copy, halo copy 0, halo copy 1 (first k-step only)
        const int npieces = 1 + APIECES + TN + (copies ? 3 : 0);
        auto piece = [&](int i) {
            if (i == 0) {
                if (last) {
                    if (more) {
#pragma unroll
                        for (int k = 0; k < TM; ++k) a_ent[k] = a_ent_n[k];
                    }
                } else if (more) {
                    read_entries(ptap_next);
                }
            } else if (i <= APIECES) {
                if (do_load) {
                    const int t0 = 2 * (i - 1);
                    load_a(nxt, t0, la, lm, lks);
                    if (t0 + 1 < TM) load_a(nxt, t0 + 1, la, lm, lks);
                }
            } else if (i <= APIECES + TN) {
                if (do_load) load_b(nxt, i - APIECES - 1, lw, lks);
            } else if (i == APIECES + TN + 1) {
                issue_w();
            } else if (i == APIECES + TN + 2) {
                issue_halo0();
            } else {
                issue_halo1();
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        __builtin_amdgcn_sched_barrier(0);
        int done = 0;
#pragma unroll
        for (int g = 0; g < GAPS; ++g) {
            mma_one(cur, g / TN, g % TN);
            __builtin_amdgcn_sched_barrier(0);
            // after matrix instruction g, as many pieces as keep them evenly spread
            const int upto = ((g + 1) * npieces + GAPS - 1) / GAPS;
            for (; done < upto && done < npieces; ++done) piece(done);
        }
        if constexpr (SPARSE) {
            // at taps 1, 4, 7: one third of the next chunk's halo, one item per lane of the whole workgroup
            if ((t == 1 || t == 4 || t == 7) && c + 1 < nchunks && !SDGP_EXP(32)) {
                const int k = t == 1 ? 0 : (t == 4 ? 1 : 2);
                const int u0 = k * hub;
                const int cnt = min(hub, nunits - u0);
                if (cnt > 0)
                    prune_items(((wave + k + c) & 7) * 64, cnt * 32, u0, off_raw + (uint32_t)((c + k) & 1) * L::kRawSlot, abuf_other,
                                mbuf_other, (uint32_t)pc_next * KC);
            }
        }
        if (last) {
            wide_wait_copies<4>();  // everything requested two stages ago has landed
            if (!SDGP_EXP(16)) __syncthreads();
            ptap_next = ptap_next + 1 == ntaps ? 0 : ptap_next + 1;
            wslot_off = wslot_next;
            if (chunk_ends) {
                t = 0, ++c;
                pc_next = pc_next + 1 == nchunks ? 0 : pc_next + 1;
                const uint32_t x = abuf; abuf = abuf_other; abuf_other = x;
                const uint32_t y = mbuf; mbuf = mbuf_other; mbuf_other = y;
            } else {
                ++t;
            }
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

    if (SDGP_EXP(1)) return;
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
