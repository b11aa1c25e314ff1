// Backward-data kernel for 1x1 convolutions without padding (any stride) and linear layers: dL/dD[rows, C_in] = prune(dL/dO)[rows, C_out] . W
// (Fig. 2; Sec. II-A).  A plain GEMM whose reduction axis is the pruned one (Fig. 1).  With C_out <= 2048 these layers
// are bound by reading dL/dO and writing dL/dD once (arithmetic intensity 50-200 FLOP/B), so the kernel is built to
// stream: a workgroup takes 128 or 256 consecutive rows and 64 to 256 columns (the host picks the shape) and walks the
// reduction in chunks of 32 channels:
//   * every byte from global memory moves with direct-to-LDS loads; the chunk after the current one is in flight
//     while the current one is multiplied (two buffers each for the gradient rows and the 32 x BN slab of W); the
//     request counter drains in front of the one barrier per chunk;
//   * pruning (Sec. III-B): the raw rows of chunk s+2 stream in while chunk s+1 is ranked / pruned / compressed (two
//     values + two 2-bit positions per aligned quad, the operand of v_smfmac_f32_32x32x32_bf16; every n <= 2 pattern
//     fits it) and chunk s is multiplied;
//   * MODE 3 takes the gradient already ranked and compressed (a pass of its own wrote, per row and 64 channels, the 32
//     kept values and their positions: csrc/compress.hip): nothing is ranked here, the reduction runs in chunks of 64
//     channels on the structured-sparse instruction, and the copies bring values and positions straight into the
//     layout the fragments are read from.  For layers where the fused kernel would rank a gradient element many
//     times over (one workgroup per column tile and per tap ranks its rows itself);
//   * wavefronts of one kind, register tiles of up to 128 x 64, two workgroups to a CU; fragments as in bwd_row.h (swizzled 16-byte
//     reads for the gradient, transpose reads for W in its native layout);
//   * the result leaves through LDS as whole rows with 16-byte stores; with a stride, a gradient pixel's row goes to
//     input pixel (p * stride, q * stride) and the other pixels of its stride x stride block receive zeros (no tap
//     reaches them).
#pragma once

#include <type_traits>

#include "lds_copy.h"

namespace sdgp {

struct PwParams {
    const uint16_t* dO;
    const uint16_t* W;
    uint16_t* dD;
    long long rows;              // GEMM rows: gradient pixels B*P*Q (gather mode: B*Pc*Qc)
    long long rows_dO;           // gradient pixels B*P*Q
    int C_out, C_in;
    int stride, P, Q, H, Wd;     // stride > 1: gradient pixel (p, q) is input pixel (p*stride, q*stride); the others get zeros
    // gather mode (one output parity class of a strided filter; see bwd_pw_plan.hip): row (b, i, j) of the class grid
    // Pc x Qc is input pixel (i*stride + oa, j*stride + ob) and sums ntaps taps; tap t reads gradient pixel
    // (i + tap_dp[t], j + tap_dq[t]) -- zeros outside the gradient -- against filter tap tap_w[t] of w_taps
    int gather, ntaps, w_taps, Pc, Qc, oa, ob;
    int tap_dp[4], tap_dq[4], tap_w[4];
    int n;
    uint32_t mix;
    int ntiles_n, nblocks;
    int idx_pitch;   // channels per gradient row in the random ranker's flat element index (C_out, or what it was before padding)
    // MODE 3: dO points at the compressed values ([rows_dO][C_out / 2] bf16) and meta at the positions
    // ([C_out / 64][rows_dO] x 8 bytes: four 16-bit words of 2-bit positions per row and 64 channels)
    const unsigned char* meta;
};

constexpr int kPwKC = 32;  // reduction channels per chunk (64 when the operand arrives compressed)

template <int BN, int MODE, int ROWS>
struct PwLayout {
    static constexpr bool kPre = MODE == 3;     // the gradient arrives ranked and compressed
    static constexpr bool kSparse = MODE == 2 || MODE == 3;
    static constexpr bool kPrunes = MODE == 1 || MODE == 2;  // raw rows are staged and ranked (MODE 1 stores them dense, zero-filled)
    static constexpr int kKC = kPre ? 64 : kPwKC;
    static constexpr int kWRow = BN * 2;
    static constexpr int kWSlab = kKC * kWRow;
    static constexpr int kWUnits = kWSlab / 1024;
    static constexpr int kAUnits = ROWS / 16;                  // 1 KB copy units (16 rows x 64 B) of a gradient chunk
    static constexpr int kABytes = ROWS * (kSparse && !kPre ? 32 : 64);  // one gradient buffer as the matrix instructions read it
    static constexpr int kRawBytes = ROWS * 64;
    static constexpr int kMetaBytes = kPre ? ROWS * 8 : kSparse ? ROWS * 4 : 0;
    static constexpr int kOutPitch = BN * 2 + 16;
    // buffer sets in the request ring: the dense kernel requests kSets - 1 chunks ahead.  Two: with three or four
    // sets the 128 x 128 dense tile drops from four workgroups per CU to two and runs 20-30 % slower -- more
    // workgroups hide the copy latency better than a deeper ring does.
    static constexpr int kSets = 2;
    static constexpr int off_w() { return 0; }
    static constexpr int off_raw() { return off_w() + kSets * kWSlab; }
    static constexpr int off_a() { return off_raw() + (kPrunes ? 2 * kRawBytes : 0); }
    static constexpr int off_meta() { return off_a() + kSets * kABytes; }
    static constexpr int loop_bytes() { return off_meta() + 2 * kMetaBytes; }
    static constexpr int out_bytes() { return ROWS * kOutPitch; }
    static constexpr int off_rowtab() { return loop_bytes() > out_bytes() ? loop_bytes() : out_bytes(); }  // strided layers only
    static constexpr int total() { return off_rowtab() + ROWS * 12; }
};

// what a tap outside the gradient copies (one 64-byte chunk row)
__device__ __align__(64) const uint32_t kPwZeros[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

template <int BN, int MODE, int M, int RK, int ROWS, int NW, bool GATHER>
__device__ __forceinline__ void bwd_pw_body(const PwParams& p) {
    using L = PwLayout<BN, MODE, ROWS>;
    static_assert(L::total() <= 160 * 1024, "LDS budget");
    constexpr bool SPARSE = L::kSparse;
    constexpr bool PRUNES = L::kPrunes;
    constexpr bool PRE = L::kPre;
    constexpr int KC = L::kKC;
    constexpr int WAVES_N = BN / 64;
    constexpr int WAVES_M = NW / WAVES_N;
    constexpr int NT = NW * 64;
    constexpr int WM = ROWS / WAVES_M;
    constexpr int TM = WM / 32;
    constexpr int TN = 2;
    static_assert(WAVES_M >= 1 && TM >= 1 && TM * 32 * WAVES_M == ROWS, "row tiles");
    constexpr int KSTEP = SPARSE ? 32 : 16;
    constexpr int NKS = KC / KSTEP;
    constexpr int CPR = BN / 8;                 // 16-byte columns per W row
    // Swizzle of the W slab: the 16-byte column of row r sits at column ^ (WSW * (r & 3)).  One pass of a transpose read
    // takes rows r .. r+3 and four columns of each; with 64 banks of 4 bytes a row of 256 bytes or more starts at bank 0,
    // so the four rows must land in four different quarters of the 256-byte bank window (WSW = 4); a 128-byte row
    // alternates between the two halves of the window by itself and only needs its halves told apart (WSW = 2).
    constexpr int WSW = BN >= 128 ? 4 : 2;
    constexpr int RPU = 1024 / L::kWRow > 0 ? 1024 / L::kWRow : 1;  // W rows per copy unit (BN <= 256: at least two)
    constexpr int WU = L::kWUnits;
    constexpr int AU = L::kAUnits;

    extern __shared__ __align__(16) unsigned char smem_generic[];
    SDGP_LDS unsigned char* smem = (SDGP_LDS unsigned char*)smem_generic;
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // consecutive logical ids stay on one XCD (workgroups are dealt round-robin over 8 XCDs): the column tiles of one
    // row tile then find the gradient rows in that XCD's L2
    int lid = blockIdx.x;
    {
        const int per = p.nblocks >> 3;
        if (lid < (per << 3)) lid = (lid & 7) * per + (lid >> 3);
    }
    const int ntile = lid % p.ntiles_n;
    const long long m0 = (long long)(lid / p.ntiles_n) * ROWS;
    const int n0 = ntile * BN;
    const int nchunks = p.C_out / KC;
    const int nstages = GATHER ? nchunks * p.ntaps : nchunks;   // reduction steps: (tap, chunk), the chunks of a tap in a row
    const long long last_row = p.rows - 1;
    const long long last_pix = (long long)p.rows_dO - 1;
    SDGP_LDS int* rowtab = (SDGP_LDS int*)(smem + L::off_rowtab());
    auto tap_of = [&](int st) { return GATHER ? (st >= nchunks) + (st >= 2 * nchunks) + (st >= 3 * nchunks) : 0; };
    const unsigned char* const gdO = reinterpret_cast<const unsigned char*>(p.dO);
    const unsigned char* const gWb = reinterpret_cast<const unsigned char*>(p.W);
    const uint32_t rowB = PRE ? (uint32_t)p.C_out : (uint32_t)p.C_out * 2u;  // bytes per gradient row (half of them when compressed)
    const uint32_t wrowB = (uint32_t)p.C_in * 2u * (uint32_t)p.w_taps;  // bytes per W row (all taps of one output channel)

    // ---- copies.  Gradient: unit u = rows 16u .. 16u+15 of the tile, 64 bytes each; LDS position (lane & 3) of row
    // (lane >> 2) holds the swizzled source column.  Rows past the tensor re-read the last row (never stored).
    const uint32_t c16_a = PRUNES ? (uint32_t)(((lane & 3) ^ ((lane >> 4) & 1)) * 16)
                                  : (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) * 16);
    // `st` below is the reduction step: tap st / nchunks, chunk st % nchunks
    // W: unit u = rows u*RPU .. of the KC x BN slab of a chunk, columns swizzled for the transpose reads.
    // The units a wavefront copies are wave, wave + NW, ...: without a row table their addresses are a per-lane base
    // (computed once) plus a wave-uniform step per reduction step, so a copy costs one 64-bit addition.  The W units of
    // one wavefront are NW * RPU rows apart, a multiple of four, so they share the lane's swizzled column.
    constexpr int APW = AU / NW;   // gradient units per wavefront and chunk
    constexpr int MPW = (ROWS / 32 + NW - 1) / NW;   // units of position words (32 rows each)
    // With a row table: the gradient pixel each of this lane's rows reads for tap t, or -1 where the tap falls outside
    // the gradient (filled once the table is built) -- a copy then needs no table read.
    int a_src[APW][4], m_src[PRE ? MPW : 1][4];
    const unsigned char* a_base[APW];
    const unsigned char* w_base = nullptr;
    const size_t w_unit_step = (size_t)(NW * RPU) * wrowB, w_chunk_step = (size_t)KC * wrowB;
    static_assert((NW * RPU) % 4 == 0, "the units of a wavefront share the swizzle");
    if constexpr (!GATHER) {
#pragma unroll
        for (int j = 0; j < APW; ++j) {
            long long row = m0 + (wave + j * NW) * 16 + (lane >> 2);
            if (row > last_row) row = last_row;
            a_base[j] = gdO + ((size_t)row * rowB + c16_a);
        }
    }
    {
        // (tap 0 of chunk 0; a gathered class adds its tap's column block per step)
        const int row = wave * RPU + lane / CPR;
        const int lchunk = (lane % CPR) ^ (WSW * (row & 3));
        int col = n0 + lchunk * 8;
        if (col > p.C_in - 8) col = p.C_in - 8;
        w_base = gWb + ((size_t)row * wrowB + (size_t)col * 2u);
    }
    // unit wave + j * NW of reduction step `st` into the buffer that starts at `dst`
    auto copy_a_j = [&](int j, int st, uint32_t dst) {
        const int u = wave + j * NW;
        if constexpr (!GATHER) {
            lds_copy16(a_base[j] + (size_t)st * 64u, dst + (uint32_t)u * 1024u);
        } else {
            const int t = tap_of(st), chunk = st - t * nchunks;
            const int src = t == 0 ? a_src[j][0] : t == 1 ? a_src[j][1] : t == 2 ? a_src[j][2] : a_src[j][3];
            const unsigned char* a = src >= 0 ? gdO + ((size_t)src * rowB + (size_t)chunk * 64u + c16_a)
                                              : reinterpret_cast<const unsigned char*>(kPwZeros) + c16_a;
            lds_copy16(a, dst + (uint32_t)u * 1024u);
        }
    };
    auto w_src_j = [&](int j, int st) {
        if constexpr (!GATHER) {
            return w_base + ((size_t)j * w_unit_step + (size_t)st * w_chunk_step);
        } else {
            const int t = tap_of(st), chunk = st - t * nchunks;
            return w_base + ((size_t)j * w_unit_step + (size_t)chunk * w_chunk_step + (size_t)(p.tap_w[t] * p.C_in) * 2u);
        }
    };
    // Dense: the W slab travels through registers (an ordinary 16-byte load per lane, stored to the same LDS position
    // a direct copy would fill) while the gradient rows take the direct path, so the two halves of a chunk's bytes use
    // two different ways into LDS.
    constexpr bool WREG = MODE == 0;
    constexpr int WPW = WU / NW;   // W units per wavefront and chunk
    u32x4_t wreg[WPW];
    auto fetch_w = [&](int st) {
#pragma unroll
        for (int j = 0; j < WPW; ++j) wreg[j] = *reinterpret_cast<const u32x4_t*>(w_src_j(j, st));
    };
    auto store_w = [&](int set) {
#pragma unroll
        for (int j = 0; j < WPW; ++j)
            *(SDGP_LDS u32x4_t*)(smem + L::off_w() + set * L::kWSlab + (wave + j * NW) * 1024 + lane * 16) = wreg[j];
    };
    // MODE 3: the positions of 32 rows per unit (8 bytes each, one 4-byte word per lane)
    // (the same for the position words: unit wave + j * NW covers 32 rows, a step is one chunk's array of all rows)
    const unsigned char* m_base[MPW];
    const size_t m_chunk_step = (size_t)p.rows_dO * 8u;
    if constexpr (PRE && !GATHER) {
#pragma unroll
        for (int j = 0; j < MPW; ++j) {
            long long row = m0 + (wave + j * NW) * 32 + (lane >> 1);
            if (row > last_row) row = last_row;
            m_base[j] = p.meta + ((size_t)row * 8u + (uint32_t)(lane & 1) * 4u);
        }
    }
    // everything chunk `chunk` needs, into buffer set `set` (pruning: the gradient goes to raw slot `set`)
    auto copy_chunk = [&](int chunk, int set, bool with_w) {
        const uint32_t a_dst = smem_base + (PRUNES ? L::off_raw() + set * L::kRawBytes : L::off_a() + set * L::kABytes);
#pragma unroll
        for (int j = 0; j < APW; ++j) copy_a_j(j, chunk, a_dst);
        if constexpr (PRE) {
            static_assert((ROWS / 32) % NW == 0, "every wavefront copies the same number of position units");
#pragma unroll
            for (int j = 0; j < MPW; ++j) {
                const int i = wave + j * NW;
                const uint32_t dst = smem_base + L::off_meta() + set * L::kMetaBytes + (uint32_t)i * 256u;
                if constexpr (!GATHER) {
                    lds_copy4(m_base[j] + (size_t)chunk * m_chunk_step, dst);
                } else {
                    const int t = tap_of(chunk), ch = chunk - t * nchunks;   // (`chunk` is the reduction step here)
                    const int src = t == 0 ? m_src[j][0] : t == 1 ? m_src[j][1] : t == 2 ? m_src[j][2] : m_src[j][3];
                    const uint32_t word = (uint32_t)(lane & 1) * 4u;
                    const unsigned char* a = src >= 0 ? p.meta + (((size_t)ch * (size_t)p.rows_dO + (size_t)src) * 8u + word)
                                                      : reinterpret_cast<const unsigned char*>(kPwZeros) + word;
                    lds_copy4(a, dst);
                }
            }
        }
        if (with_w) {
#pragma unroll
            for (int j = 0; j < WPW; ++j)
                lds_copy16(w_src_j(j, chunk), smem_base + L::off_w() + set * L::kWSlab + (uint32_t)(wave + j * NW) * 1024u);
        }
    };
    auto copy_w_chunk = [&](int chunk, int set) {
#pragma unroll
        for (int j = 0; j < WPW; ++j)
            lds_copy16(w_src_j(j, chunk), smem_base + L::off_w() + set * L::kWSlab + (uint32_t)(wave + j * NW) * 1024u);
    };

    // rank / prune / compress raw slot `set` (chunk `chunk`) into gradient buffer `set`: ROWS * 2 items of 16 channels
    auto prune_chunk = [&](int chunk, int set) {
        if constexpr (PRUNES && !SPARSE) {
            // any n of m (m up to 32): the pruned rows are stored dense, zeros in the dropped positions, in the layout
            // the dense matrix instruction reads.  One item = one m-group or sixteen channels, whichever is larger.
            constexpr int IC = M > 16 ? M : 16;       // channels per item
            constexpr int IPR = KC / IC;              // items per row of the chunk
#pragma unroll 1
            for (int item = tid; item < ROWS * IPR; item += NT) {
                const int row = item / IPR, part = item % IPR;
                SDGP_LDS unsigned char* src = smem + L::off_raw() + set * L::kRawBytes + row * 64;
                SDGP_LDS unsigned char* dst = smem + L::off_a() + set * L::kABytes + row * 64;
                const int sw = (row >> 2) & 1, sw2 = (row >> 2) & 3;
                if constexpr (RK != kRandom && (M == 16 || M == 32)) {
                    // one group per item, magnitude keys: the packed 16-bit ranker (ranker.h), no unpacking
                    uint32_t wv[IC / 2], ov[IC / 2];
#pragma unroll
                    for (int g = 0; g < IC / 8; ++g) {
                        const u32x4_t v = *(SDGP_LDS u32x4_t*)(src + (((part * (IC / 8) + g) ^ sw) * 16));
                        wv[4 * g] = v[0], wv[4 * g + 1] = v[1], wv[4 * g + 2] = v[2], wv[4 * g + 3] = v[3];
                    }
                    prune_packed<M, RK>(wv, p.n, ov);
#pragma unroll
                    for (int g = 0; g < IC / 8; ++g) {
                        const u32x4_t x = {ov[4 * g], ov[4 * g + 1], ov[4 * g + 2], ov[4 * g + 3]};
                        *(SDGP_LDS u32x4_t*)(dst + (((part * (IC / 8) + g) ^ sw2) << 4)) = x;
                    }
                    continue;
                }
                uint32_t raw[IC], out[IC];
#pragma unroll
                for (int g = 0; g < IC / 8; ++g) {
                    const u32x4_t v = *(SDGP_LDS u32x4_t*)(src + (((part * (IC / 8) + g) ^ sw) * 16));
#pragma unroll
                    for (int x = 0; x < 4; ++x) raw[g * 8 + 2 * x] = v[x] & 0xFFFFu, raw[g * 8 + 2 * x + 1] = v[x] >> 16;
                }
                uint64_t e0 = 0;
                if constexpr (RK == kRandom) {
                    const int t = tap_of(chunk), ch = chunk - t * nchunks;  // (`chunk` is the reduction step here)
                    long long grow = m0 + row;
                    if constexpr (GATHER) grow = (long long)rowtab[3 * row] + (long long)p.tap_dp[t] * p.Q + p.tap_dq[t];
                    grow = grow < 0 ? 0 : (grow > last_pix ? last_pix : grow);
                    e0 = (uint64_t)grow * (uint64_t)p.idx_pitch + (uint64_t)(ch * KC + part * IC);
                }
#pragma unroll
                for (int g = 0; g < IC / M; ++g) {
                    uint32_t r[M], o[M];
                    bool kk[M];
#pragma unroll
                    for (int j = 0; j < M; ++j) r[j] = raw[g * M + j];
                    const uint64_t eg = e0 + (uint64_t)(g * M);
                    prune_group<kBF16, M, RK, false>(r, p.n, hash_row(p.mix, (uint32_t)(eg >> 32)), (uint32_t)eg, kk, o);
#pragma unroll
                    for (int j = 0; j < M; ++j) out[g * M + j] = o[j];
                }
#pragma unroll
                for (int g = 0; g < IC / 8; ++g) {
                    const u32x4_t x = {out[g * 8] | (out[g * 8 + 1] << 16), out[g * 8 + 2] | (out[g * 8 + 3] << 16),
                                       out[g * 8 + 4] | (out[g * 8 + 5] << 16), out[g * 8 + 6] | (out[g * 8 + 7] << 16)};
                    *(SDGP_LDS u32x4_t*)(dst + (((part * (IC / 8) + g) ^ sw2) << 4)) = x;
                }
            }
        }
        if constexpr (SPARSE && PRUNES) {
#pragma unroll 1
            for (int item = tid; item < ROWS * 2; item += NT) {
                const int row = item >> 1, part = item & 1;
                SDGP_LDS unsigned char* src = smem + L::off_raw() + set * L::kRawBytes + row * 64;
                const int sw = (row >> 2) & 1;
                u32x4_t v[2];
                v[0] = *(SDGP_LDS u32x4_t*)(src + (((2 * part) ^ sw) * 16));
                v[1] = *(SDGP_LDS u32x4_t*)(src + (((2 * part + 1) ^ sw) * 16));
                uint64_t e0 = 0;
                if constexpr (RK == kRandom) {
                    const int t = tap_of(chunk), ch = chunk - t * nchunks;  // (`chunk` is the reduction step here)
                    long long grow = m0 + row;
                    if constexpr (GATHER) grow = (long long)rowtab[3 * row] + (long long)p.tap_dp[t] * p.Q + p.tap_dq[t];
                    grow = grow < 0 ? 0 : (grow > last_pix ? last_pix : grow);  // (rows of zeros: any index will do)
                    e0 = (uint64_t)grow * (uint64_t)p.idx_pitch + (uint64_t)(ch * KC + part * 16);
                }
                uint32_t packed[4], meta;
                prune16_compressed<M, RK>(v, p.n, p.mix, e0, packed, meta);
                const u32x4_t x = {packed[0], packed[1], packed[2], packed[3]};
                *(SDGP_LDS u32x4_t*)(smem + L::off_a() + set * L::kABytes + row * 32 + part * 16) = x;
                *(SDGP_LDS uint16_t*)(smem + L::off_meta() + set * L::kMetaBytes + row * 4 + part * 2) = (uint16_t)meta;
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

    // ---- prologue
    if constexpr (GATHER) {
        // per row of the tile: flat index of gradient pixel (b, i, j) (it may lie outside the gradient: the taps add
        // their shifts), i and j, and the input pixel the row is stored to
        for (int m = tid; m < ROWS; m += NT) {
            const long long row = m0 + m;
            int base = -1, ij = 0, opix = -1;
            if (row <= last_row) {
                const int pq = p.Pc * p.Qc;
                const int b = (int)(row / pq), rem = (int)(row - (long long)b * pq);
                const int i = rem / p.Qc, j = rem - i * p.Qc;
                base = (b * p.P + i) * p.Q + j;
                if (base < 0) base = 0;
                ij = i | (j << 16);
                opix = (b * p.H + i * p.stride + p.oa) * p.Wd + j * p.stride + p.ob;
            }
            rowtab[3 * m] = base, rowtab[3 * m + 1] = ij, rowtab[3 * m + 2] = opix;
        }
        __syncthreads();
        auto tap_source = [&](int rl, int t) {
            const int base = rowtab[3 * rl], ij = rowtab[3 * rl + 1];
            const int i = (ij & 0xFFFF) + p.tap_dp[t], j = (ij >> 16) + p.tap_dq[t];
            const bool ok = t < p.ntaps && base >= 0 && i >= 0 && i < p.P && j >= 0 && j < p.Q;
            long long src = (long long)base + (long long)p.tap_dp[t] * p.Q + p.tap_dq[t];
            src = src < 0 ? 0 : (src > last_pix ? last_pix : src);  // (a valid tap is inside anyway)
            return ok ? (int)src : -1;
        };
#pragma unroll
        for (int j = 0; j < APW; ++j)
#pragma unroll
            for (int t = 0; t < 4; ++t) a_src[j][t] = tap_source((wave + j * NW) * 16 + (lane >> 2), t);
        if constexpr (PRE) {
#pragma unroll
            for (int j = 0; j < MPW; ++j)
#pragma unroll
                for (int t = 0; t < 4; ++t) m_src[j][t] = tap_source((wave + j * NW) * 32 + (lane >> 1), t);
        }
    }
    constexpr int SETS = L::kSets;
    static_assert(AU % NW == 0 && WU % NW == 0, "every wavefront issues the same number of copies per chunk");
    constexpr int kCopiesPerChunk = AU / NW + WU / NW;
    if constexpr (PRUNES) {
        copy_chunk(0, 0, true);
        if (nstages > 1) copy_chunk(1, 1, false);
        wait_lds_copies<0>();
        __syncthreads();
        prune_chunk(0, 0);
    } else if constexpr (WREG) {
        static_assert(SETS == 2, "one chunk ahead");
        copy_chunk(0, 0, false);
        fetch_w(0);
        store_w(0);
    } else {
#pragma unroll
        for (int i = 0; i < SETS - 1; ++i)
            if (i < nstages) copy_chunk(i, i, true);
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
    const uint32_t half = (uint32_t)(lane >> 5);
    uint32_t a_lane[TM];  // this lane's row of each row tile inside a gradient buffer (swizzle included)
    uint32_t m_lane[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        const uint32_t row = (uint32_t)(wm * WM + t * 32 + (lane & 31));
        a_lane[t] = SPARSE && !PRE ? row * 32u + half * 16u : row * 64u + (((half ^ (row >> 2)) & 3u) << 4);
        m_lane[t] = PRE ? row * 8u + half * 2u : row * 4u + half * 2u;
    }
    struct Frags {
        u32x4_t a[TM];
        int meta[TM];
        typename std::conditional<SPARSE, bf16x16_t, bf16x8_t>::type b[TN];
    };
    auto load_frags = [&](Frags& f, int set, int ks) {
#pragma unroll
        for (int t = 0; t < TM; ++t) {
            if constexpr (PRE) {
                f.a[t] = *(SDGP_LDS u32x4_t*)(smem + L::off_a() + set * L::kABytes + (a_lane[t] ^ (uint32_t)(ks * 32)));
                f.meta[t] = *(SDGP_LDS uint16_t*)(smem + L::off_meta() + set * L::kMetaBytes + m_lane[t] + ks * 4);
            } else if constexpr (SPARSE) {
                f.a[t] = *(SDGP_LDS u32x4_t*)(smem + L::off_a() + set * L::kABytes + a_lane[t]);
                f.meta[t] = *(SDGP_LDS uint16_t*)(smem + L::off_meta() + set * L::kMetaBytes + m_lane[t]);
            } else {
                f.a[t] = *(SDGP_LDS u32x4_t*)(smem + L::off_a() + set * L::kABytes + (a_lane[t] ^ (uint32_t)(ks * 32)));
            }
        }
#pragma unroll
        for (int u = 0; u < TN; ++u) {
            SDGP_LDS unsigned char* wb = smem + b_lane[u] + set * L::kWSlab;
            if constexpr (SPARSE) {
                s16x4_t q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    q[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SDGP_LDS s16x4_t*)(wb + (ks * 32 + (i >> 1) * 16 + (i & 1) * 4) * L::kWRow));
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
        }
    };
    auto mma = [&](const Frags& f) {
#pragma unroll
        for (int t = 0; t < TM; ++t) {
            const bf16x8_t a = __builtin_bit_cast(bf16x8_t, f.a[t]);
#pragma unroll
            for (int u = 0; u < TN; ++u) {
                if constexpr (SPARSE)
                    acc[t][u] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, f.b[u], acc[t][u], f.meta[t], 0, 0);
                else
                    acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, f.b[u], acc[t][u], 0, 0, 0);
            }
        }
    };

    // ---- main loop: one chunk per stage
    Frags fr[2];
    int set = 0, set_req = SETS - 1;  // dense: ring positions of chunk s and of the chunk requested during stage s
    for (int s = 0; s < nstages; ++s) {
        if constexpr (PRUNES) set = s & 1;
        // requests for what comes next: dense -- chunk s + SETS - 1 into the set that the previous stage read;
        // pruning -- W of chunk s+1 and the raw rows of chunk s+2 (into the slot whose rows were ranked during the
        // previous stage)
        if constexpr (PRUNES) {
            if (s + 1 < nstages) copy_w_chunk(s + 1, set ^ 1);
            if (s + 2 < nstages) {
                const uint32_t a_dst = smem_base + L::off_raw() + set * L::kRawBytes;
#pragma unroll
                for (int j = 0; j < APW; ++j) copy_a_j(j, s + 2, a_dst);
            }
        } else {
            if (s + SETS - 1 < nstages) {
                copy_chunk(s + SETS - 1, set_req, !WREG);
                if constexpr (WREG) fetch_w(s + SETS - 1);
            }
        }
        load_frags(fr[0], set, 0);
        if constexpr (PRUNES) {
            if (s + 1 < nstages) prune_chunk(s + 1, set ^ 1);  // its raw rows landed before the last barrier
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            if (ks + 1 < NKS) load_frags(fr[(ks + 1) & 1], set, ks + 1);
            __builtin_amdgcn_sched_barrier(0);
            mma(fr[ks & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (PRUNES) {
            wait_lds_copies<0>();
        } else {
            // chunk s + 1 has to be there; the requests of the chunks after it (issued in order, the same number by
            // every wavefront) may stay in flight.  Near the end fewer are outstanding: drain.
            if constexpr (WREG) {
                if (s + 1 < nstages) store_w(set_req);   // (its last readers passed the barrier that ended the previous stage)
                wait_lds_copies<0>();
            } else {
                if (s + SETS - 1 < nstages) wait_lds_copies<(SETS - 2) * kCopiesPerChunk>();
                else wait_lds_copies<0>();
            }
            set = set + 1 == SETS ? 0 : set + 1;
            set_req = set_req + 1 == SETS ? 0 : set_req + 1;
        }
        __syncthreads();
    }

    // ---- epilogue: fp32 -> bf16 (RNE) into LDS, then whole rows with 16-byte stores
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
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
                *(SDGP_LDS uint16_t*)(smem + m * L::kOutPitch + col * 2) = (uint16_t)pk;
                *(SDGP_LDS uint16_t*)(smem + (m + 1) * L::kOutPitch + col * 2) = (uint16_t)(pk >> 16);
            }
    if (!GATHER && p.stride > 1) {
        // where each row of the tile goes: its input pixel and how many of the stride x stride pixels it owns exist
        for (int m = tid; m < ROWS; m += NT) {
            const long long row = m0 + m;
            int pix = -1, lim = 0;
            if (row <= last_row) {
                const int pq = p.P * p.Q;
                const int b = (int)(row / pq), rem = (int)(row - (long long)b * pq);
                const int pp = rem / p.Q, qq = rem - pp * p.Q;
                const int h = pp * p.stride, w = qq * p.stride;
                pix = (b * p.H + h) * p.Wd + w;
                lim = (min(p.stride, p.H - h) << 8) | min(p.stride, p.Wd - w);
            }
            rowtab[2 * m] = pix, rowtab[2 * m + 1] = lim;
        }
    }
    __syncthreads();
    if (!GATHER && p.stride == 1) {
#pragma unroll 4
        for (int idx = tid; idx < ROWS * CPR; idx += NT) {
            const int m = idx / CPR, cc = idx % CPR;
            const long long row = m0 + m;
            if (row <= last_row && n0 + cc * 8 < p.C_in) {
                const u32x4_t v = *(SDGP_LDS u32x4_t*)(smem + m * L::kOutPitch + cc * 16);
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p.dD + (size_t)row * p.C_in + n0 + cc * 8));
            }
        }
    } else if (GATHER) {
        for (int idx = tid; idx < ROWS * CPR; idx += NT) {
            const int m = idx / CPR, cc = idx % CPR;
            const int pix = rowtab[3 * m + 2];
            if (pix >= 0 && n0 + cc * 8 < p.C_in) {
                const u32x4_t v = *(SDGP_LDS u32x4_t*)(smem + m * L::kOutPitch + cc * 16);
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p.dD + (size_t)pix * p.C_in + n0 + cc * 8));
            }
        }
    } else {
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        for (int idx = tid; idx < ROWS * CPR; idx += NT) {
            const int m = idx / CPR, cc = idx % CPR;
            const int pix = rowtab[2 * m], lim = rowtab[2 * m + 1];
            if (pix >= 0 && n0 + cc * 8 < p.C_in) {
                const u32x4_t v = *(SDGP_LDS u32x4_t*)(smem + m * L::kOutPitch + cc * 16);
                uint16_t* dst = p.dD + (size_t)pix * p.C_in + n0 + cc * 8;
                const int ny = lim >> 8, nx = lim & 255;
                for (int dy = 0; dy < ny; ++dy)
                    for (int dx = 0; dx < nx; ++dx)
                        __builtin_nontemporal_store((dy | dx) ? zero : v, reinterpret_cast<u32x4_t*>(dst + (size_t)(dy * p.Wd + dx) * p.C_in));
            }
        }
    }
}

// One problem per launch.
template <int BN, int MODE, int M, int RK, int ROWS, int NW, bool GATHER>
__global__ void __launch_bounds__(NW * 64) bwd_pw(const PwParams p) {
    bwd_pw_body<BN, MODE, M, RK, ROWS, NW, GATHER>(p);
}

// The parity classes of one strided filter in one launch: blockIdx.y is the class, blockIdx.x the tile of that class
// (the grid is as wide as the largest class).  The classes are small GEMMs, often less than one round of workgroups
// each; side by side, one class's last workgroups run beside the next one's first.
constexpr int kPwMaxClasses = 16;
struct PwClasses {
    PwParams c[kPwMaxClasses];
};

template <int BN, int MODE, int M, int RK, int ROWS, int NW>
__global__ void __launch_bounds__(NW * 64) bwd_pw_classes(const PwClasses all) {
    const PwParams& p = all.c[blockIdx.y];
    if ((int)blockIdx.x >= p.nblocks) return;
    bwd_pw_body<BN, MODE, M, RK, ROWS, NW, true>(p);
}

}  // namespace sdgp
