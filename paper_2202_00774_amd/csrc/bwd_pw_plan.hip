// Host side of the pointwise kernel: 1x1 convolutions without padding (any stride) and linear layers whose channel
// counts fit (C_out a multiple of 32, C_in a multiple of 8); chooses the tile shape and launches.
#include <climits>

#include "bwd_pw_launch.h"

namespace sdgp {

int launch_pw_dense(const PwParams& p, int shape, hipStream_t stream);
int launch_pw_sparse_m4(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_sparse_m8(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_sparse_m16(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_masked_m4(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_masked_m8(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_masked_m16(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_masked_m32(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_classes_dense(const PwClasses& all, int ncls, int shape, hipStream_t stream);
int launch_pw_classes_sparse_m4(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream);
int launch_pw_classes_sparse_m8(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream);
int launch_pw_classes_sparse_m16(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream);
int launch_pw_classes_masked_m4(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream);
int launch_pw_classes_masked_m8(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream);
int launch_pw_classes_masked_m16(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream);
int launch_pw_classes_masked_m32(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream);
int launch_pw_pre(const PwParams& p, int shape, hipStream_t stream);
int launch_pw_classes_pre(const PwClasses& all, int ncls, int shape, hipStream_t stream);
size_t compress_meta_offset(int64_t rows, int64_t C_out);
size_t compress_bytes(int64_t rows, int64_t C_out);
int compress_launch(const void* dO, int64_t rows, int64_t C_out, int n, int m, int rk, uint64_t seed, void* workspace,
                    hipStream_t stream);

namespace {

// 0: dense (n == m); 2: at most two survivors per aligned quad, the structured-sparse instruction; 1: any other n of
// m in {4, 8, 16, 32}, pruned rows stored dense with zeros; -1: not for this kernel
int pw_mode(int n, int m) {
    if (n == m) return 0;
    if (n <= 2 && (m == 4 || m == 8 || m == 16)) return 2;
    if (m == 4 || m == 8 || m == 16 || m == 32) return 1;
    return -1;
}

int launch_pw_any(const PwParams& p, int mode, int m, int shape, int rk, hipStream_t stream) {
    if (mode == 0) return launch_pw_dense(p, shape, stream);
    if (mode == 2) {
        if (m == 4) return launch_pw_sparse_m4(p, shape, rk, stream);
        if (m == 8) return launch_pw_sparse_m8(p, shape, rk, stream);
        return launch_pw_sparse_m16(p, shape, rk, stream);
    }
    if (m == 4) return launch_pw_masked_m4(p, shape, rk, stream);
    if (m == 8) return launch_pw_masked_m8(p, shape, rk, stream);
    if (m == 16) return launch_pw_masked_m16(p, shape, rk, stream);
    return launch_pw_masked_m32(p, shape, rk, stream);
}

int launch_pw_classes_any(const PwClasses& all, int ncls, int mode, int m, int shape, int rk, hipStream_t stream) {
    if (mode == 0) return launch_pw_classes_dense(all, ncls, shape, stream);
    if (mode == 2) {
        if (m == 4) return launch_pw_classes_sparse_m4(all, ncls, shape, rk, stream);
        if (m == 8) return launch_pw_classes_sparse_m8(all, ncls, shape, rk, stream);
        return launch_pw_classes_sparse_m16(all, ncls, shape, rk, stream);
    }
    if (m == 4) return launch_pw_classes_masked_m4(all, ncls, shape, rk, stream);
    if (m == 8) return launch_pw_classes_masked_m8(all, ncls, shape, rk, stream);
    if (m == 16) return launch_pw_classes_masked_m16(all, ncls, shape, rk, stream);
    return launch_pw_classes_masked_m32(all, ncls, shape, rk, stream);
}

// Tile shape of the fused and dense kernels.  Workgroups of four wavefronts, two or more to a CU, so that one's loads
// and stores overlap the other's arithmetic.  Pruning: all of C_in (up to 256 columns) in one workgroup, so every
// gradient row is ranked once per 256 columns; dense: 128 x 128 tiles measured fastest (column tiles of one row tile
// run side by side on one XCD and find the gradient rows in its L2).
int pw_shape(int mode, int64_t C_in, int64_t C_out) {
    if (C_in <= 64) return 3;   // 128 x 64: 256-row tiles measured the same or slower (fewer workgroups, a longer last round)
    if (mode != 0 && C_in > 128 && C_out > 64) return 0;   // (64 channels to rank: ranking them per 128 columns costs less than the third workgroup per CU gains)
    return 1;
}
// Tile shape when the gradient arrives compressed (nothing is ranked in the kernel): the dense kernel's.
int pw_pre_shape(int64_t C_in) { return C_in <= 64 ? 3 : 1; }

// Whether a pass that ranks and compresses the gradient first (csrc/compress.hip) pays: the fused kernel would rank
// every gradient element `times` times, the pass reads it once and writes half of it, and the product that follows
// runs 1.15-1.25 times as fast as the dense one.  Measured on the layers of ResNet-50 at batch 256: from two times on
// with the random ranker (the hash makes ranking dearer), from four on with the magnitude rankers.
bool pre_pays(int mode, int64_t C_out, int64_t rows_dO, int times, int rk) {
    const int least = rk == kRandom ? 2 : 4;
    return mode == 2 && (C_out % 64) == 0 && times >= least && rows_dO * (C_out / 16) < ((int64_t)1 << 31);
}

struct PwPlan {
    PwParams p;
    int mode, shape;
    bool pre;       // rank and compress first, then MODE 3 (needs the workspace)
    size_t bytes;   // workspace of the pre path
};

// 0 and the plan, or 1 when the pointwise kernel does not take the problem.
int pw_plan(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n, int m,
            int rk, PwPlan& out, int force_shape = -1) {
    const int mode = pw_mode(n, m);
    if (mode < 0) return 1;
    if (R != 1 || S != 1 || stride < 1 || stride > 255 || pad != 0 || (C_out % kPwKC) != 0 || (C_in % 8) != 0) return 1;
    if (mode != 0 && (C_out % m) != 0) return 1;
    const int64_t P = (H - 1) / stride + 1, Q = (Wd - 1) / stride + 1;  // gradient image
    const int64_t rows = B * P * Q;
    if (stride > 1 && (B * H * Wd >= INT_MAX || H < 1 || Wd < 1)) return 1;
    if (rows < 1 || C_out < kPwKC || C_in < 8 || C_out >= (1 << 24) || C_in >= (1 << 24)) return 1;

    PwParams p{};
    p.rows = rows, p.C_out = (int)C_out, p.C_in = (int)C_in, p.idx_pitch = (int)C_out;
    p.n = n;
    p.stride = stride, p.P = (int)P, p.Q = (int)Q, p.H = (int)H, p.Wd = (int)Wd;
    p.rows_dO = rows, p.gather = 0, p.ntaps = 1, p.w_taps = 1;

    int shape = force_shape >= 0 ? force_shape : pw_shape(mode, C_in, C_out);
    const int fused_tiles_n = (int)((C_in + kPwShapes[shape].bn - 1) / kPwShapes[shape].bn);
    out.pre = force_shape < 0 && pre_pays(mode, C_out, rows, fused_tiles_n, rk);
    if (out.pre) shape = pw_pre_shape(C_in);
    const int bn = kPwShapes[shape].bn, rows_per = kPwShapes[shape].rows;
    const int64_t blocks = ((rows + rows_per - 1) / rows_per) * ((C_in + bn - 1) / bn);
    // too small to be worth a matrix-core launch of this shape (a forced shape: the caller has decided)
    if ((blocks < 64 && force_shape < 0) || blocks < 1 || blocks >= INT_MAX) return 1;
    p.ntiles_n = (int)((C_in + bn - 1) / bn);
    p.nblocks = (int)blocks;
    out.p = p, out.mode = mode, out.shape = shape;
    out.bytes = out.pre ? compress_bytes(rows, C_out) : 0;
    return 0;
}

// ---- small 1x1 / linear problems whose C_out is a multiple of 8 but not of the chunk (a classifier's 1000 outputs):
// the gradient rows and the filter are copied into the workspace with C_out rounded up to the chunk, zeros in the new
// channels, and the kernel runs on the copies.  Zero channels change nothing: a group of zeros keeps zeros, a zero
// filter row adds nothing, and the random ranker's element index keeps the original row pitch.
typedef uint32_t pad_u32x4 __attribute__((ext_vector_type(4)));

// dst [rows][vout] <- src [rows][vin] 16-byte vectors, zero where the column is new
__global__ void __launch_bounds__(256) pad_columns(const pad_u32x4* __restrict__ src, pad_u32x4* __restrict__ dst, int64_t total,
                                                   int vin, int vout) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int64_t r = i / vout;
    const int c = (int)(i - r * vout);
    dst[i] = c < vin ? src[r * vin + c] : pad_u32x4{0u, 0u, 0u, 0u};
}
// dst [nout] <- src [nin] 16-byte vectors, zeros after them
__global__ void __launch_bounds__(256) pad_tail(const pad_u32x4* __restrict__ src, pad_u32x4* __restrict__ dst, int64_t nin,
                                                int64_t nout) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= nout) return;
    dst[i] = i < nin ? src[i] : pad_u32x4{0u, 0u, 0u, 0u};
}

struct PadPlan {
    int64_t rows, Kp;
    size_t off_w, bytes;
};
// Whether the padded path takes the problem (and its workspace): plain 1x1 stride 1, at most 16 M elements in either copy.
bool pad_plan(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n, int m,
              PadPlan& out) {
    if (R != 1 || S != 1 || stride != 1 || pad != 0) return false;
    if (C_out < kPwKC || (C_out % kPwKC) == 0 || (C_out % 8) != 0 || (C_in % 8) != 0 || C_in < 8) return false;
    if (pw_mode(n, m) < 0 || (n != m && (C_out % m) != 0)) return false;
    const int64_t rows = B * H * Wd, Kp = (C_out + kPwKC - 1) / kPwKC * kPwKC;
    if (rows < 1 || rows * Kp > ((int64_t)1 << 24) || Kp * C_in > ((int64_t)1 << 24)) return false;
    out.rows = rows, out.Kp = Kp;
    out.off_w = ((size_t)rows * (size_t)Kp * 2u + 255u) & ~(size_t)255u;
    out.bytes = out.off_w + (size_t)Kp * (size_t)C_in * 2u;
    return true;
}

}  // namespace

// Workspace bytes with which bwd_pw_launch / bwd_gather_launch rank the gradient once, in a pass of their own (0: the
// fused kernel is used, or neither takes the problem).
size_t bwd_pw_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n,
                        int m);

// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.  With a
// workspace of at least bwd_pw_workspace(...) bytes the gradient is ranked once, in a pass of its own, where that
// pays; with less the fused kernel runs.
int bwd_pw_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                  int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed, void* workspace, size_t workspace_bytes,
                  hipStream_t stream) {
    if (!is_aligned16(dO) || !is_aligned16(W) || !is_aligned16(dD)) return 1;
    PadPlan padded{};
    if (pad_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, padded)) {
        if (workspace == nullptr || workspace_bytes < padded.bytes || !is_aligned16(workspace)) return 1;  // another kernel takes it
        PwPlan plan{};
        const int shape = 3;   // 128 x 64 tiles, the most workgroups: these problems are small
        if (pw_plan(1, 1, padded.rows, C_in, padded.Kp, 1, 1, 1, 0, n, m, rk, plan, shape) != 0) return 1;
        PwParams& p = plan.p;
        p.idx_pitch = (int)C_out;
        pad_u32x4* dOp = static_cast<pad_u32x4*>(workspace);
        pad_u32x4* Wp = reinterpret_cast<pad_u32x4*>(static_cast<unsigned char*>(workspace) + padded.off_w);
        const int64_t n_dO = padded.rows * (padded.Kp / 8), n_w_in = C_out * (C_in / 8), n_w_out = padded.Kp * (C_in / 8);
        hipLaunchKernelGGL(pad_columns, dim3((unsigned)((n_dO + 255) / 256)), dim3(256), 0, stream, static_cast<const pad_u32x4*>(dO), dOp,
                           n_dO, (int)(C_out / 8), (int)(padded.Kp / 8));
        hipLaunchKernelGGL(pad_tail, dim3((unsigned)((n_w_out + 255) / 256)), dim3(256), 0, stream, static_cast<const pad_u32x4*>(W), Wp,
                           n_w_in, n_w_out);
        if (launch_status() != SDGP_OK) return SDGP_ERR_HIP;
        p.dO = reinterpret_cast<const uint16_t*>(dOp);
        p.W = reinterpret_cast<const uint16_t*>(Wp);
        p.dD = static_cast<uint16_t*>(dD);
        p.mix = seed_mix(seed);
        return launch_pw_any(p, plan.mode, m, shape, rk, stream);
    }
    PwPlan plan{};
    if (pw_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, rk, plan) != 0) return 1;
    if (plan.pre && (workspace == nullptr || workspace_bytes < plan.bytes || !is_aligned16(workspace))) {
        // no room for the compressed gradient: the fused kernel
        const int shape = pw_shape(plan.mode, C_in, C_out);
        const int bn = kPwShapes[shape].bn, rows_per = kPwShapes[shape].rows;
        const int64_t blocks = ((plan.p.rows + rows_per - 1) / rows_per) * ((C_in + bn - 1) / bn);
        if (blocks < 64 || blocks >= INT_MAX) return 1;
        plan.p.ntiles_n = (int)((C_in + bn - 1) / bn), plan.p.nblocks = (int)blocks;
        plan.shape = shape, plan.pre = false;
    }
    PwParams& p = plan.p;
    p.W = static_cast<const uint16_t*>(W);
    p.dD = static_cast<uint16_t*>(dD);
    p.mix = seed_mix(seed);
    if (plan.pre) {
        const int rc = compress_launch(dO, p.rows_dO, C_out, n, m, rk, seed, workspace, stream);
        if (rc != SDGP_OK) return rc;
        p.dO = static_cast<const uint16_t*>(workspace);
        p.meta = static_cast<const unsigned char*>(workspace) + compress_meta_offset(p.rows_dO, C_out);
        return launch_pw_pre(p, plan.shape, stream);
    }
    p.dO = static_cast<const uint16_t*>(dO);
    return launch_pw_any(p, plan.mode, m, plan.shape, rk, stream);
}

// Strided filters wider than 1x1 (the stride-2 3x3 layers of a ResNet): the input pixels split into stride x stride
// parity classes; class (a, b) -- pixels (i*stride + a, j*stride + b) -- is a small stride-1 correlation over the
// gradient with the taps r = a + pad (mod stride), s = b + pad (mod stride), at most four of them here.  Each class is
// a GEMM of the pointwise kernel whose reduction runs over (tap, channel) and whose rows are gathered from the gradient
// pixels (i + dp, j + dq) of each tap, zeros outside; all classes go out in one launch (blockIdx.y = class).  Each
// gradient element is ranked once per tap that reads it (the kept set does not depend on who asks).
namespace {

struct GatherPlan {
    PwClasses all;
    int ncls, mode, shape;
    bool pre;
    size_t bytes;
};

// 0 and the plan for the shape the fused kernels use (pre == false) or the compressed-operand kernel uses, or 1.
int gather_plan(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n, int m,
                bool want_pre, GatherPlan& out) {
    const int mode = pw_mode(n, m);
    if (mode < 0) return 1;
    if (stride < 2 || stride > 4 || R < stride || S < stride || R > 2 * stride || S > 2 * stride || pad < 0) return 1;
    if (C_out < kPwKC || (C_out % kPwKC) != 0 || C_in < 8 || (C_in % 8) != 0) return 1;
    if (mode != 0 && (C_out % m) != 0) return 1;
    if (H + 2 * pad < R || Wd + 2 * pad < S || H < stride || Wd < stride) return 1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    if (B < 1 || P < 1 || Q < 1 || P >= 65536 || Q >= 32768 || H >= 65536 || Wd >= 32768 || B * (P + 8) * (Q + 8) >= (1 << 30) || B * H * Wd >= INT_MAX ||
        C_out >= (1 << 20) || (int64_t)R * S * C_in >= (1 << 20))
        return 1;

    PwParams base{};
    base.C_out = (int)C_out, base.C_in = (int)C_in, base.idx_pitch = (int)C_out;
    base.n = n;
    base.stride = stride, base.P = (int)P, base.Q = (int)Q, base.H = (int)H, base.Wd = (int)Wd;
    base.rows_dO = B * P * Q, base.gather = 1, base.w_taps = R * S;

    // every tap of every class ranks the rows it reads: R * S times per gradient element and column tile
    out.pre = want_pre && pre_pays(mode, C_out, base.rows_dO, R * S, kRandom);
    const int shape = out.pre ? pw_pre_shape(C_in) : pw_shape(mode, C_in, C_out);
    const int bn = kPwShapes[shape].bn, rows_per = kPwShapes[shape].rows;
    base.ntiles_n = (int)((C_in + bn - 1) / bn);

    // all classes first: nothing is launched unless every one of them fits
    static_assert(kPwMaxClasses >= 16, "stride up to four");
    PwParams* cls = out.all.c;
    int ncls = 0;
    for (int a = 0; a < stride; ++a)
        for (int b = 0; b < stride; ++b) {
            PwParams q = base;
            q.oa = a, q.ob = b;
            q.Pc = (int)((H - a + stride - 1) / stride), q.Qc = (int)((Wd - b + stride - 1) / stride);
            q.ntaps = 0;
            for (int r = 0; r < R; ++r) {
                if ((a + pad - r) % stride != 0) continue;
                for (int sx = 0; sx < S; ++sx) {
                    if ((b + pad - sx) % stride != 0) continue;
                    if (q.ntaps == 4) return 1;
                    q.tap_dp[q.ntaps] = (a + pad - r) / stride, q.tap_dq[q.ntaps] = (b + pad - sx) / stride;
                    q.tap_w[q.ntaps] = r * S + sx;
                    ++q.ntaps;
                }
            }
            if (q.ntaps == 0) return 1;
            q.rows = B * q.Pc * q.Qc;
            const int64_t blocks = ((q.rows + rows_per - 1) / rows_per) * q.ntiles_n;
            if (q.rows < 1 || blocks < 64 || blocks >= INT_MAX) return 1;
            q.nblocks = (int)blocks;
            cls[ncls++] = q;
        }
    // classes with more taps first: their workgroups run longest, and the launch should end on the short ones
    for (int i = 1; i < ncls; ++i)
        for (int j = i; j > 0 && cls[j].ntaps > cls[j - 1].ntaps; --j) {
            const PwParams t = cls[j];
            cls[j] = cls[j - 1];
            cls[j - 1] = t;
        }
    out.ncls = ncls, out.mode = mode, out.shape = shape;
    out.bytes = out.pre ? compress_bytes(base.rows_dO, C_out) : 0;
    return 0;
}

}  // namespace

// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.  Workspace as
// for bwd_pw_launch.
int bwd_gather_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                      int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed, void* workspace, size_t workspace_bytes,
                      hipStream_t stream) {
    if (!is_aligned16(dO) || !is_aligned16(W) || !is_aligned16(dD)) return 1;
    GatherPlan plan{};
    bool planned = false;
    if (workspace != nullptr && is_aligned16(workspace)) {
        planned = gather_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, true, plan) == 0 && (!plan.pre || workspace_bytes >= plan.bytes);
    }
    if (!planned && gather_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, false, plan) != 0) return 1;
    const int64_t rows_dO = plan.all.c[0].rows_dO;
    const void* grad = dO;
    const unsigned char* meta = nullptr;
    if (plan.pre) {
        const int rc = compress_launch(dO, rows_dO, C_out, n, m, rk, seed, workspace, stream);
        if (rc != SDGP_OK) return rc;
        grad = workspace;
        meta = static_cast<const unsigned char*>(workspace) + compress_meta_offset(rows_dO, C_out);
    }
    for (int i = 0; i < plan.ncls; ++i) {
        PwParams& q = plan.all.c[i];
        q.dO = static_cast<const uint16_t*>(grad), q.meta = meta;
        q.W = static_cast<const uint16_t*>(W), q.dD = static_cast<uint16_t*>(dD);
        q.mix = seed_mix(seed);
    }
    if (plan.pre) return launch_pw_classes_pre(plan.all, plan.ncls, plan.shape, stream);
    return launch_pw_classes_any(plan.all, plan.ncls, plan.mode, m, plan.shape, rk, stream);
}

size_t bwd_pw_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int n,
                        int m) {
    PadPlan padded{};
    if (pad_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, padded)) return padded.bytes;
    PwPlan one{};
    // (the ranker that takes the pass soonest: the size is enough for any)
    if (pw_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, kRandom, one) == 0) return one.bytes;
    GatherPlan many{};
    if (gather_plan(B, H, Wd, C_in, C_out, R, S, stride, pad, n, m, true, many) == 0) return many.bytes;
    return 0;
}

}  // namespace sdgp
