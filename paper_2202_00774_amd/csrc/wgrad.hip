// Weight gradient of a convolution layer (Sec. II-A, Fig. 1):
//   dW[k,r,s,c] = sum_{b,p,q} dO[b,p,q,k] * D[b, p*stride + r - pad, q*stride + s - pad, c]
// from the UNPRUNED output gradient (Sec. III-A: dO is kept for this product, the data gradient gets a pruned copy).
//
// Matrix-core kernel (bf16, stride 1, 3x3): the reduction runs over pixels, so both operands of
// v_mfma_f32_32x32x16_bf16 take "16 pixels" as their K dimension: A = dO^T (32 output channels x 16 pixels),
// B = D shifted by the tap (16 pixels x 32 input channels).  Both tiles sit in LDS as [pixel][channel], the way they
// sit in memory, and ds_read_b64_tr_b16 hands each lane one channel for four consecutive pixels.
//   * a workgroup (4 wavefronts, one per SIMD, up to 512 registers each) owns a block of 64*TM output channels x 64
//     input channels x 9 taps and walks over tiles of TR gradient rows of one image; wavefront w takes output
//     channels (w&1)*32*TM .. and input channels (w>>1)*32 ..: TM x 9 accumulator tiles, 2*(TM+9) fragment reads per
//     9*TM matrix instructions;
//   * the next tile travels global -> registers while the current one is multiplied, then registers -> LDS;
//   * workgroups that share an output block split the tiles between them and write fp32 partial blocks to the
//     workspace; a second kernel adds the partials in a fixed order, so the result does not depend on timing.
// Everything else (other filters, strides, channel counts, fp32) goes to a plain reduction kernel.
#include "common.h"

namespace sdgp {

namespace {

#define SDGP_LDS __attribute__((address_space(3)))
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kCB = 64;               // input channels per workgroup
constexpr int kPitchB = kCB * 2 + 32; // bytes per pixel of the D tile: four consecutive pixels fall into disjoint banks
constexpr int kMaxTilePixels = 128;
constexpr int kMaxUnitsA = 8;         // 16-byte units per thread of the dO tile: 128 pixels x 128 channels
constexpr int kMaxUnitsB = 8;         // and of the D tile (at most 256 halo pixels x 64 channels)

struct WgradParams {
    const uint16_t* D;
    const uint16_t* dO;
    float* partial;       // [nsplit][C_out][R][S][C_in]
    int64_t nW;
    int64_t total_tiles;  // B * tiles_per_image, or ceil(B / NI)
    int64_t B;
    int H, Wd, P, Q, C_in, C_out, pad;
    int TR, TP, TP16;     // gradient rows per tile, its pixels, rounded up to 16
    int tiles_per_image;
    int NI;               // images per tile: more than one only when a tile holds whole images (TR == P)
    int hrows, hw;        // rows and width of one image's part of the D tile: TR + R - 1, Q + S - 1
    int cblocks;          // C_in / 64
    int nsplit;
};

template <int TM>
struct WgradLayout {
    static constexpr int kKB = 64 * TM;
    static constexpr int kPitchA = kKB * 2 + 32;
    __host__ __device__ static int off_b(int tp16) { return tp16 * kPitchA; }
    __host__ __device__ static int off_tab(int tp16, int hp) { return off_b(tp16) + hp * kPitchB; }
    __host__ __device__ static int off_hrc(int tp16, int hp) { return off_tab(tp16, hp) + tp16 * 4; }
    __host__ __device__ static int total(int tp16, int hp) { return off_hrc(tp16, hp) + hp * 4; }
};

template <int R, int S, int TM>
__global__ void __launch_bounds__(kThreads) wgrad_mfma(WgradParams p) {
    using L = WgradLayout<TM>;
    constexpr int KB = L::kKB, NT = R * S;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x;
    const int kb = blockIdx.y / p.cblocks, cb = blockIdx.y % p.cblocks;
    const int hpi = p.hrows * p.hw, hp = p.NI * hpi;
    unsigned char* const tileA = smem;
    unsigned char* const tileB = smem + L::off_b(p.TP16);
    int* const hoff = reinterpret_cast<int*>(smem + L::off_tab(p.TP16, hp));
    int* const hrc = reinterpret_cast<int*>(smem + L::off_hrc(p.TP16, hp));   // image << 24 | row << 12 | column of a D-tile pixel

    // byte offset of tile pixel j inside the D tile (tap (0,0)); pixels past the tile's end meet zero gradient rows
    for (int j = tid; j < p.TP16; j += kThreads) {
        const int jj = j < p.TP ? j : 0;
        const int ii = jj / (p.TR * p.Q), in = jj % (p.TR * p.Q);
        hoff[j] = ((ii * p.hrows + in / p.Q) * p.hw + in % p.Q) * kPitchB;
    }
    for (int j = tid; j < hp; j += kThreads) hrc[j] = ((j / hpi) << 24) | (((j % hpi) / p.hw) << 12) | ((j % hpi) % p.hw);
    __syncthreads();

    const int unitsA = p.TP16 * (KB / 8), unitsB = hp * (kCB / 8);
    u32x4_t ra[kMaxUnitsA], rb[kMaxUnitsB];

    auto fetch = [&](int64_t tile) {   // global -> registers
        const int64_t b = p.NI > 1 ? tile * p.NI : tile / p.tiles_per_image;     // first image of the tile
        const int p0 = p.NI > 1 ? 0 : (int)(tile % p.tiles_per_image) * p.TR;
        // gradient pixels of this tile that exist: whole images up to the batch's end, or rows up to the image's end
        const int live = p.NI > 1 ? (int)(p.B - b < p.NI ? p.B - b : p.NI) * p.TR * p.Q
                                  : (p.P - p0 < p.TR ? p.P - p0 : p.TR) * p.Q;
        const uint16_t* const srcA = p.dO + ((b * p.P + p0) * p.Q) * (int64_t)p.C_out + kb * KB;
#pragma unroll
        for (int i = 0; i < kMaxUnitsA; ++i) {
            const int u = tid + i * kThreads;
            const int pix = u / (KB / 8), col = u % (KB / 8);
            ra[i] = u32x4_t{0u, 0u, 0u, 0u};
            if (pix < live) ra[i] = *reinterpret_cast<const u32x4_t*>(srcA + pix * (int64_t)p.C_out + col * 8);
        }
#pragma unroll
        for (int i = 0; i < kMaxUnitsB; ++i) {
            const int u = tid + i * kThreads;
            rb[i] = u32x4_t{0u, 0u, 0u, 0u};
            if (u < unitsB) {
                const int hpix = u / (kCB / 8), col = u % (kCB / 8);
                const int rc = hrc[hpix];
                const int64_t bi = b + (rc >> 24);
                const int h = p0 + ((rc >> 12) & 0xFFF) - p.pad, w = (rc & 0xFFF) - p.pad;
                if (bi < p.B && h >= 0 && h < p.H && w >= 0 && w < p.Wd)
                    rb[i] = *reinterpret_cast<const u32x4_t*>(p.D + ((bi * p.H + h) * (int64_t)p.Wd + w) * p.C_in + cb * kCB + col * 8);
            }
        }
    };
    auto stage = [&]() {               // registers -> LDS
#pragma unroll
        for (int i = 0; i < kMaxUnitsA; ++i) {
            const int u = tid + i * kThreads;
            if (u < unitsA) *reinterpret_cast<u32x4_t*>(tileA + (u / (KB / 8)) * L::kPitchA + (u % (KB / 8)) * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < kMaxUnitsB; ++i) {
            const int u = tid + i * kThreads;
            if (u < unitsB) *reinterpret_cast<u32x4_t*>(tileB + (u / (kCB / 8)) * kPitchB + (u % (kCB / 8)) * 16) = rb[i];
        }
    };

    // Accumulators: TM x NT tiles of 16 registers.  The first 16 tiles live in the accumulation registers, the rest
    // in ordinary ones: the matrix instruction is written as inline assembly so that the compiler cannot move a tile
    // between the two files inside the loop.
    f32x16_t acc[TM][NT];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][q][e] = 0.0f;
    auto mma = [&](int t, int q, const bf16x8_t& a, const bf16x8_t& b) {
        if (t * NT + q < 16) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[t][q]) : "v"(a), "v"(b));
        else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[t][q]) : "v"(a), "v"(b));
    };

    // lane's part of a fragment: 16-lane group g reads pixels 8*(g/2) + 4*i + (lane%16)/4 and the four channels
    // 16*(g%2) + 4*(lane%4) .. of the 32 the wavefront's tile covers
    const int g = lane >> 4, l16 = lane & 15;
    const int pix_in_step = 8 * (g >> 1) + (l16 >> 2);
    const int col = (16 * (g & 1) + 4 * (l16 & 3)) * 2;
    const int colA = ((wave & 1) * 32 * TM) * 2 + col;
    const int colB = ((wave >> 1) * 32) * 2 + col;
    const int nsteps = p.TP16 / 16;

    struct Frags {
        bf16x8_t a[TM];
        bf16x8_t b[NT];
    };
    auto tr8 = [&](const unsigned char* lo_ptr, const unsigned char* hi_ptr) {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SDGP_LDS s16x4_t*)lo_ptr);
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SDGP_LDS s16x4_t*)hi_ptr);
        const s16x8_t all = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8_t, all);
    };
    // One step = 16 pixels: TM * NT matrix instructions on fragments `cur`, with the reads of the next step's
    // fragments `nxt` spread between them (a step past the tile's end re-reads the last one and is not multiplied).
    auto step_pair = [&](const Frags& cur, Frags& nxt, int next_step) {
        const int ns = next_step < nsteps ? next_step : nsteps - 1;
        const int j0 = ns * 16 + pix_in_step, j1 = j0 + 4;
        const int h0 = hoff[j0] + colB, h1 = hoff[j1] + colB;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
#pragma unroll
            for (int t = 0; t < TM; ++t) mma(t, q, cur.a[t], cur.b[q]);
            const int tap = ((q / S) * p.hw + q % S) * kPitchB;
            nxt.b[q] = tr8(tileB + h0 + tap, tileB + h1 + tap);
            if (q < TM) nxt.a[q] = tr8(tileA + j0 * L::kPitchA + colA + q * 64, tileA + j1 * L::kPitchA + colA + q * 64);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    int64_t tile = split;
    if (tile < p.total_tiles) fetch(tile);
    for (; tile < p.total_tiles; tile += p.nsplit) {
        __syncthreads();   // every wavefront has finished reading the previous tile
        stage();
        __syncthreads();
        if (tile + p.nsplit < p.total_tiles) fetch(tile + p.nsplit);
        Frags f0, f1;
        {
            const int j0 = pix_in_step, j1 = j0 + 4;
            const int h0 = hoff[j0] + colB, h1 = hoff[j1] + colB;
#pragma unroll
            for (int t = 0; t < TM; ++t) f0.a[t] = tr8(tileA + j0 * L::kPitchA + colA + t * 64, tileA + j1 * L::kPitchA + colA + t * 64);
#pragma unroll
            for (int q = 0; q < NT; ++q) f0.b[q] = tr8(tileB + h0 + ((q / S) * p.hw + q % S) * kPitchB, tileB + h1 + ((q / S) * p.hw + q % S) * kPitchB);
        }
        for (int step = 0; step < nsteps; step += 2) {
            step_pair(f0, f1, step + 1);
            if (step + 1 < nsteps) step_pair(f1, f0, step + 2);
        }
    }
    // the matrix pipe may still be writing the last tiles: the compiler does not know these instructions' latency
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

    // result register e of lane l: output channel 8*(e/4) + 4*(l/32) + e%4, input channel l%32 of the tile
    float* const out = p.partial + (int64_t)split * p.nW;
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int k = kb * KB + (wave & 1) * 32 * TM + t * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const int c = cb * kCB + (wave >> 1) * 32 + (lane & 31);
                out[((int64_t)k * NT + q) * p.C_in + c] = acc[t][q][e];
            }
}

// dW[e] = sum of the partial filters.  A workgroup takes 64 elements; its four wavefronts each add a quarter of the
// splits (four loads in flight), then the four sums are added in wavefront order: a fixed order for a given shape.
__global__ void __launch_bounds__(kThreads) wgrad_reduce(const float* partial, float* dW, int64_t nW, int nsplit) {
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int64_t e = (int64_t)blockIdx.x * 64 + lane;
    const int per = (nsplit + 3) / 4;
    const int first = grp * per, last = first + per < nsplit ? first + per : nsplit;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    if (e < nW) {
        int i = first;
        for (; i + 3 < last; i += 4) {
            s0 += partial[(int64_t)i * nW + e];
            s1 += partial[(int64_t)(i + 1) * nW + e];
            s2 += partial[(int64_t)(i + 2) * nW + e];
            s3 += partial[(int64_t)(i + 3) * nW + e];
        }
        for (; i < last; ++i) s0 += partial[(int64_t)i * nW + e];
    }
    part[grp][lane] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (grp == 0 && e < nW) dW[e] = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
}

struct SimpleArgs {
    const void* D;
    const void* dO;
    float* dW;
    int64_t B, H, Wd, P, Q, C_in, C_out;
    int R, S, stride, pad;
};

// One workgroup per filter element: its threads stride over the output pixels, then add their sums in LDS.
template <int DT>
__global__ void __launch_bounds__(kThreads) wgrad_simple(SimpleArgs a) {
    __shared__ float part[kThreads];
    const int64_t e = blockIdx.x;
    const int64_t c = e % a.C_in, s = (e / a.C_in) % a.S, r = (e / (a.C_in * a.S)) % a.R, k = e / (a.C_in * a.S * a.R);
    const int64_t npix = a.B * a.P * a.Q;
    float acc = 0.0f;
    for (int64_t pix = threadIdx.x; pix < npix; pix += kThreads) {
        const int64_t q = pix % a.Q, pp = (pix / a.Q) % a.P, b = pix / (a.Q * a.P);
        const int64_t h = pp * a.stride + r - a.pad, w = q * a.stride + s - a.pad;
        if (h < 0 || h >= a.H || w < 0 || w >= a.Wd) continue;
        float gv, xv;
        if constexpr (DT == SDGP_BF16) {
            gv = bf16_to_float(reinterpret_cast<const uint16_t*>(a.dO)[pix * a.C_out + k]);
            xv = bf16_to_float(reinterpret_cast<const uint16_t*>(a.D)[((b * a.H + h) * a.Wd + w) * a.C_in + c]);
        } else {
            gv = reinterpret_cast<const float*>(a.dO)[pix * a.C_out + k];
            xv = reinterpret_cast<const float*>(a.D)[((b * a.H + h) * a.Wd + w) * a.C_in + c];
        }
        acc = fmaf(gv, xv, acc);
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int half = kThreads / 2; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half) part[threadIdx.x] += part[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) a.dW[e] = part[0];
}

// Filters of at most kSmallElems elements (a first layer: 64 x 3x3 x 3): a workgroup takes a run of output pixels and
// every filter element, thread i owning elements i, i + 256, ...; the gradient row and the patch of a pixel are read
// by all threads at once (one cache line each), partial filters go to the workspace like the matrix-core kernel's.
constexpr int kSmallPerThread = 8;
constexpr int kSmallElems = kSmallPerThread * kThreads;
constexpr int kSmallGroups = 1024;

template <int DT>
__global__ void __launch_bounds__(kThreads) wgrad_small(SimpleArgs a, float* partial, int64_t nW) {
    const int64_t npix = a.B * a.P * a.Q;
    const int64_t per = (npix + gridDim.x - 1) / gridDim.x;
    const int64_t first = (int64_t)blockIdx.x * per, last = first + per < npix ? first + per : npix;
    int k[kSmallPerThread], c[kSmallPerThread], r[kSmallPerThread], s[kSmallPerThread];
    float acc[kSmallPerThread];
#pragma unroll
    for (int i = 0; i < kSmallPerThread; ++i) {
        const int64_t e = threadIdx.x + i * kThreads;
        const int64_t ee = e < nW ? e : 0;
        c[i] = (int)(ee % a.C_in), s[i] = (int)((ee / a.C_in) % a.S), r[i] = (int)((ee / (a.C_in * a.S)) % a.R);
        k[i] = (int)(ee / (a.C_in * a.S * a.R));
        acc[i] = 0.0f;
    }
    for (int64_t pix = first; pix < last; ++pix) {
        const int64_t q = pix % a.Q, pp = (pix / a.Q) % a.P, b = pix / (a.Q * a.P);
#pragma unroll
        for (int i = 0; i < kSmallPerThread; ++i) {
            if (threadIdx.x + i * kThreads >= nW) continue;
            const int64_t h = pp * a.stride + r[i] - a.pad, w = q * a.stride + s[i] - a.pad;
            if (h < 0 || h >= a.H || w < 0 || w >= a.Wd) continue;
            float gv, xv;
            if constexpr (DT == SDGP_BF16) {
                gv = bf16_to_float(reinterpret_cast<const uint16_t*>(a.dO)[pix * a.C_out + k[i]]);
                xv = bf16_to_float(reinterpret_cast<const uint16_t*>(a.D)[((b * a.H + h) * a.Wd + w) * a.C_in + c[i]]);
            } else {
                gv = reinterpret_cast<const float*>(a.dO)[pix * a.C_out + k[i]];
                xv = reinterpret_cast<const float*>(a.D)[((b * a.H + h) * a.Wd + w) * a.C_in + c[i]];
            }
            acc[i] = fmaf(gv, xv, acc[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < kSmallPerThread; ++i) {
        const int64_t e = threadIdx.x + i * kThreads;
        if (e < nW) partial[(int64_t)blockIdx.x * nW + e] = acc[i];
    }
}

bool small_filter(int64_t nW, int64_t npix) { return nW > 0 && nW <= kSmallElems && npix >= 4 * kSmallGroups; }

// Layers with few input channels (a first layer, R*S*C_in of 27 or 147) and 64 or 128 output channels.  A workgroup
// walks over segments of up to 64 pixels of one gradient row, with the segment's gradient values (fp32 [pixel][k]) and
// the R image rows it touches in LDS.  Thread (k = tid % 64, g = tid / 64) owns filter elements (k, t) and (k + 64, t)
// for t = g, g + 4, ... of the R*S*C_in patch positions: per pixel one gradient read per output channel and one
// patch read per position (the same address in every lane of a wavefront), one FMA each.
constexpr int kNarrowPix = 64;
constexpr int kNarrowMaxT = 148;                  // 7 x 7 x 3 and below
constexpr int kNarrowGroups = 1024;

struct NarrowArgs {
    const uint16_t* D;
    const uint16_t* dO;
    float* partial;                   // [gridDim.x][C_out * T]
    int64_t B, segments;
    int H, Wd, P, Q, C_in, C_out, R, S, stride, pad;
    int T, SC, rowlen, qsegs;
    uint32_t cin_magic;               // ceil(2^16 / C_in): x / C_in == (x * magic) >> 16 for the x of a staged row
};

template <int KB, int kNarrowSlots>   // C_out / 64; patch positions per thread: 4 * kNarrowSlots >= R*S*C_in
__global__ void __launch_bounds__(kThreads) wgrad_narrow(NarrowArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* const gl = lds;                                  // [64 pixels][64 * KB]
    float* const halo = lds + kNarrowPix * 64 * KB;         // [R][rowlen]
    const int tid = threadIdx.x, k = tid & 63, g = tid >> 6;
    int off[kNarrowSlots];                                  // where patch position t = g + 4 i sits for pixel 0
    float acc[KB][kNarrowSlots];
#pragma unroll
    for (int i = 0; i < kNarrowSlots; ++i) {
        const int t = g + 4 * i, tt = t < a.T ? t : 0;
        off[i] = (tt / a.SC) * a.rowlen + tt % a.SC;
#pragma unroll
        for (int u = 0; u < KB; ++u) acc[u][i] = 0.0f;
    }
    for (int64_t seg = blockIdx.x; seg < a.segments; seg += gridDim.x) {
        const int q0 = (int)(seg % a.qsegs) * kNarrowPix;
        const int p = (int)((seg / a.qsegs) % a.P);
        const int64_t b = seg / ((int64_t)a.qsegs * a.P);
        const int npx = a.Q - q0 < kNarrowPix ? a.Q - q0 : kNarrowPix;
        __syncthreads();
        for (int e = tid; e < kNarrowPix * 64 * KB; e += kThreads) {
            const int px = e / (64 * KB), kk = e % (64 * KB);
            gl[e] = px < npx ? bf16_to_float(a.dO[((b * a.P + p) * (int64_t)a.Q + q0 + px) * a.C_out + kk]) : 0.0f;
        }
        for (int r = 0; r < a.R; ++r) {
            const int h = p * a.stride + r - a.pad;
            const uint16_t* const src = a.D + ((b * a.H + h) * (int64_t)a.Wd + q0 * a.stride - a.pad) * a.C_in;
            for (int x = tid; x < a.rowlen; x += kThreads) {
                const int w = q0 * a.stride - a.pad + (int)(((uint32_t)x * a.cin_magic) >> 16);
                halo[r * a.rowlen + x] = (h >= 0 && h < a.H && w >= 0 && w < a.Wd) ? bf16_to_float(src[x]) : 0.0f;
            }
        }
        __syncthreads();
        for (int px = 0; px < npx; ++px) {
            float gv[KB];
#pragma unroll
            for (int u = 0; u < KB; ++u) gv[u] = gl[px * 64 * KB + u * 64 + k];
            const float* const patch = halo + px * a.stride * a.C_in;
#pragma unroll
            for (int i = 0; i < kNarrowSlots; ++i) {   // a slot past the patch's end repeats position 0 and is not stored
                const float xv = patch[off[i]];
#pragma unroll
                for (int u = 0; u < KB; ++u) acc[u][i] = fmaf(gv[u], xv, acc[u][i]);
            }
        }
    }
    float* const out = a.partial + (int64_t)blockIdx.x * a.C_out * a.T;
#pragma unroll
    for (int i = 0; i < kNarrowSlots; ++i) {
        const int t = g + 4 * i;
        if (t < a.T) {
#pragma unroll
            for (int u = 0; u < KB; ++u) out[(int64_t)(k + 64 * u) * a.T + t] = acc[u][i];
        }
    }
}

bool narrow_layer(int64_t C_in, int64_t C_out, int R, int S, int stride, int dt, int64_t H, int64_t Wd) {
    const int64_t T = (int64_t)R * S * C_in;
    if (dt != SDGP_BF16 || T > kNarrowMaxT || (C_out != 64 && C_out != 128) || C_in >= 32) return false;
    if (H > (1 << 24) || Wd > (1 << 24)) return false;
    const int64_t rowlen = ((kNarrowPix - 1) * stride + S) * C_in;
    const size_t lds = ((size_t)kNarrowPix * C_out + (size_t)R * rowlen) * sizeof(float);
    return lds <= 150 * 1024 && rowlen <= 2048;
}

struct Plan {
    bool mfma;
    int TM, TR, NI, TP, TP16, tiles_per_image, hrows, hw, cblocks, kblocks, nsplit, lds;
    int64_t total_tiles;
};

// The matrix-core kernel takes bf16, stride 1, 3x3 with pad <= 2, C_in % 64 == 0, C_out % 64 == 0 and rows of at most
// 128 gradient pixels; everything else goes to the reduction kernel.
Plan make_plan(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt) {
    Plan pl{};
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    if (dt != SDGP_BF16 || stride != 1 || R != 3 || S != 3 || C_in % 64 != 0 || C_out % 64 != 0 || C_in == 0 || C_out == 0)
        return pl;
    if (B <= 0 || P <= 0 || Q <= 0 || Q > kMaxTilePixels || H > (1 << 20) || Wd > (1 << 20) || B > ((int64_t)1 << 31)) return pl;
    pl.TM = (C_out % 128 == 0) ? 2 : 1;
    pl.TR = (int)(kMaxTilePixels / Q);
    if (pl.TR > P) pl.TR = (int)P;
    pl.hw = (int)Q + S - 1;
    while (pl.TR > 1 && (pl.TR + R - 1) * pl.hw * (kCB / 8) > kMaxUnitsB * kThreads) --pl.TR;
    pl.hrows = pl.TR + R - 1;
    if (pl.hrows * pl.hw * (kCB / 8) > kMaxUnitsB * kThreads) return pl;
    if (pl.hrows > 4095 || pl.hw > 4095) return pl;
    pl.NI = 1;
    if (pl.TR == P)  // small images: several per tile, as many as the tile's pixel and halo limits allow
        while (pl.NI < B && (pl.NI + 1) * P * Q <= kMaxTilePixels && (pl.NI + 1) * pl.hrows * pl.hw * (kCB / 8) <= kMaxUnitsB * kThreads)
            ++pl.NI;
    pl.TP = pl.NI * pl.TR * (int)Q;
    pl.TP16 = (pl.TP + 15) & ~15;
    pl.tiles_per_image = (int)((P + pl.TR - 1) / pl.TR);
    pl.total_tiles = pl.NI > 1 ? (B + pl.NI - 1) / pl.NI : B * pl.tiles_per_image;
    pl.cblocks = (int)(C_in / kCB);
    pl.kblocks = (int)(C_out / (64 * pl.TM));
    const int blocks = pl.cblocks * pl.kblocks;
    int64_t ns = (256 + blocks - 1) / blocks;          // one workgroup per compute unit
    if (ns > pl.total_tiles) ns = pl.total_tiles;
    if (ns < 1) ns = 1;
    pl.nsplit = (int)ns;
    const int hp = pl.NI * pl.hrows * pl.hw;
    pl.lds = pl.TM == 2 ? WgradLayout<2>::total(pl.TP16, hp) : WgradLayout<1>::total(pl.TP16, hp);
    if (pl.lds > 160 * 1024 || blocks > 65535) return pl;
    pl.mfma = true;
    return pl;
}

}  // namespace

size_t wgrad_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt) {
    const Plan pl = make_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, dt);
    const int64_t nW = C_out * R * S * C_in;
    if (pl.mfma) return (size_t)pl.nsplit * (size_t)nW * sizeof(float);
    const int64_t npix = B * ((H + 2 * pad - R) / stride + 1) * ((Wd + 2 * pad - S) / stride + 1);
    if (npix > 0 && narrow_layer(C_in, C_out, R, S, stride, dt, H, Wd)) return (size_t)kNarrowGroups * (size_t)nW * sizeof(float);
    if (small_filter(nW, npix)) return (size_t)kSmallGroups * (size_t)nW * sizeof(float);
    return 0;
}

int wgrad_launch(const void* D, const void* dO, float* dW, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                 int R, int S, int stride, int pad, int dt, void* workspace, hipStream_t stream) {
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    const int64_t nW = C_out * R * S * C_in;
    if (nW == 0) return SDGP_OK;
    const Plan pl = make_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, dt);
    if (pl.mfma && workspace != nullptr) {
        WgradParams p{};
        p.D = (const uint16_t*)D, p.dO = (const uint16_t*)dO, p.partial = (float*)workspace;
        p.nW = nW, p.total_tiles = pl.total_tiles, p.B = B, p.NI = pl.NI;
        p.H = (int)H, p.Wd = (int)Wd, p.P = (int)P, p.Q = (int)Q, p.C_in = (int)C_in, p.C_out = (int)C_out, p.pad = pad;
        p.TR = pl.TR, p.TP = pl.TP, p.TP16 = pl.TP16, p.tiles_per_image = pl.tiles_per_image;
        p.hrows = pl.hrows, p.hw = pl.hw, p.cblocks = pl.cblocks, p.nsplit = pl.nsplit;
        const dim3 grid((unsigned)pl.nsplit, (unsigned)(pl.cblocks * pl.kblocks));
        hipError_t err;
        if (pl.TM == 2) {
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_mfma<3, 3, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, pl.lds);
            if (err != hipSuccess) return SDGP_ERR_HIP;
            wgrad_mfma<3, 3, 2><<<grid, kThreads, pl.lds, stream>>>(p);
        } else {
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_mfma<3, 3, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, pl.lds);
            if (err != hipSuccess) return SDGP_ERR_HIP;
            wgrad_mfma<3, 3, 1><<<grid, kThreads, pl.lds, stream>>>(p);
        }
        if (hipGetLastError() != hipSuccess) return SDGP_ERR_HIP;
        const int64_t blocks = (nW + 63) / 64;
        wgrad_reduce<<<(unsigned)blocks, kThreads, 0, stream>>>((const float*)workspace, dW, nW, pl.nsplit);
        return launch_status();
    }
    if (nW > 0x7FFFFFFF) return SDGP_ERR_SHAPE;
    SimpleArgs a{D, dO, dW, B, H, Wd, P, Q, C_in, C_out, R, S, stride, pad};
    if (workspace != nullptr && !pl.mfma && B * P * Q > 0 && narrow_layer(C_in, C_out, R, S, stride, dt, H, Wd)) {
        NarrowArgs n{};
        n.D = (const uint16_t*)D, n.dO = (const uint16_t*)dO, n.partial = (float*)workspace, n.B = B;
        n.H = (int)H, n.Wd = (int)Wd, n.P = (int)P, n.Q = (int)Q, n.C_in = (int)C_in, n.C_out = (int)C_out;
        n.R = R, n.S = S, n.stride = stride, n.pad = pad;
        n.T = R * S * (int)C_in, n.SC = S * (int)C_in;
        n.rowlen = ((kNarrowPix - 1) * stride + S) * (int)C_in;
        n.qsegs = (int)((Q + kNarrowPix - 1) / kNarrowPix);
        n.segments = B * P * n.qsegs;
        n.cin_magic = (65536u + (uint32_t)C_in - 1) / (uint32_t)C_in;
        const size_t lds = ((size_t)kNarrowPix * C_out + (size_t)R * n.rowlen) * sizeof(float);
        // every workgroup writes its partial filter, so the grid is fixed: the reduction reads kNarrowGroups of them
        const bool few = n.T <= 28;
        void (*kernel)(NarrowArgs) = C_out == 64 ? (few ? wgrad_narrow<1, 7> : wgrad_narrow<1, 37>)
                                                 : (few ? wgrad_narrow<2, 7> : wgrad_narrow<2, 37>);
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SDGP_ERR_HIP;
        kernel<<<kNarrowGroups, kThreads, lds, stream>>>(n);
        if (hipGetLastError() != hipSuccess) return SDGP_ERR_HIP;
        wgrad_reduce<<<(unsigned)((nW + 63) / 64), kThreads, 0, stream>>>((const float*)workspace, dW, nW, kNarrowGroups);
        return launch_status();
    }
    if (workspace != nullptr && !pl.mfma && small_filter(nW, B * P * Q)) {
        if (dt == SDGP_BF16) wgrad_small<SDGP_BF16><<<kSmallGroups, kThreads, 0, stream>>>(a, (float*)workspace, nW);
        else wgrad_small<SDGP_F32><<<kSmallGroups, kThreads, 0, stream>>>(a, (float*)workspace, nW);
        if (hipGetLastError() != hipSuccess) return SDGP_ERR_HIP;
        wgrad_reduce<<<(unsigned)((nW + 63) / 64), kThreads, 0, stream>>>((const float*)workspace, dW, nW, kSmallGroups);
        return launch_status();
    }
    if (dt == SDGP_BF16) wgrad_simple<SDGP_BF16><<<(unsigned)nW, kThreads, 0, stream>>>(a);
    else wgrad_simple<SDGP_F32><<<(unsigned)nW, kThreads, 0, stream>>>(a);
    return launch_status();
}

}  // namespace sdgp
