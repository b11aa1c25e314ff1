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

}  // namespace

// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.
int bwd_pw_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                  int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed, hipStream_t stream) {
    const int mode = pw_mode(n, m);
    if (mode < 0) return 1;
    if (R != 1 || S != 1 || stride < 1 || stride > 255 || pad != 0 || (C_out % kPwKC) != 0 || (C_in % 8) != 0) return 1;
    if (mode != 0 && (C_out % m) != 0) return 1;
    if (!is_aligned16(dO) || !is_aligned16(W) || !is_aligned16(dD)) return 1;
    const int64_t P = (H - 1) / stride + 1, Q = (Wd - 1) / stride + 1;  // gradient image
    const int64_t rows = B * P * Q;
    if (stride > 1 && (B * H * Wd >= INT_MAX || H < 1 || Wd < 1)) return 1;
    if (rows < 1 || C_out < kPwKC || C_in < 8 || C_out >= (1 << 24) || C_in >= (1 << 24)) return 1;

    PwParams p{};
    p.dO = static_cast<const uint16_t*>(dO);
    p.W = static_cast<const uint16_t*>(W);
    p.dD = static_cast<uint16_t*>(dD);
    p.rows = rows, p.C_out = (int)C_out, p.C_in = (int)C_in;
    p.n = n;
    p.stride = stride, p.P = (int)P, p.Q = (int)Q, p.H = (int)H, p.Wd = (int)Wd;
    p.rows_dO = rows, p.gather = 0, p.ntaps = 1, p.w_taps = 1;
    p.mix = seed_mix(seed);

    // tile shape.  Workgroups of four wavefronts, two to a CU, so that one's loads and stores overlap the other's
    // arithmetic.  Pruning: all of C_in (up to 256 columns) in one workgroup, so every gradient row is ranked once;
    // dense: 128 x 128 tiles measured fastest (column tiles of one row tile run side by side on one XCD and find
    // the gradient rows in its L2).
    auto blocks_of = [&](int rows_per, int bn) { return ((rows + rows_per - 1) / rows_per) * ((C_in + bn - 1) / bn); };
    int shape;
    if (C_in <= 64) shape = (mode != 0) ? 3 : 2;
    else if (mode != 0 && C_in > 128) shape = 0;
    else shape = 1;
    const int bn = kPwShapes[shape].bn, rows_per = kPwShapes[shape].rows;
    const int64_t blocks = blocks_of(rows_per, bn);
    if (blocks < 64 || blocks >= INT_MAX) return 1;  // too small to be worth a matrix-core launch of this shape
    p.ntiles_n = (int)((C_in + bn - 1) / bn);
    p.nblocks = (int)blocks;

    return launch_pw_any(p, mode, m, shape, rk, stream);
}

// Strided filters wider than 1x1 (the stride-2 3x3 layers of a ResNet): the input pixels split into stride x stride
// parity classes; class (a, b) -- pixels (i*stride + a, j*stride + b) -- is a small stride-1 correlation over the
// gradient with the taps r = a + pad (mod stride), s = b + pad (mod stride), at most four of them here.  Each class is
// a GEMM of the pointwise kernel whose reduction runs over (tap, channel) and whose rows are gathered from the gradient
// pixels (i + dp, j + dq) of each tap, zeros outside; all classes go out in one launch (blockIdx.y = class).  Each
// gradient element is ranked once per tap that reads it (the kept set does not depend on who asks).
// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.
int bwd_gather_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                      int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed, hipStream_t stream) {
    const int mode = pw_mode(n, m);
    if (mode < 0) return 1;
    if (stride < 2 || stride > 4 || R < stride || S < stride || R > 2 * stride || S > 2 * stride || pad < 0) return 1;
    if (C_out < kPwKC || (C_out % kPwKC) != 0 || C_in < 8 || (C_in % 8) != 0) return 1;
    if (mode != 0 && (C_out % m) != 0) return 1;
    if (!is_aligned16(dO) || !is_aligned16(W) || !is_aligned16(dD)) return 1;
    if (H + 2 * pad < R || Wd + 2 * pad < S || H < stride || Wd < stride) return 1;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    if (B < 1 || P < 1 || Q < 1 || P >= 65536 || Q >= 32768 || H >= 65536 || Wd >= 32768 || B * (P + 8) * (Q + 8) >= (1 << 30) || B * H * Wd >= INT_MAX ||
        C_out >= (1 << 20) || (int64_t)R * S * C_in >= (1 << 20))
        return 1;

    PwParams base{};
    base.dO = static_cast<const uint16_t*>(dO);
    base.W = static_cast<const uint16_t*>(W);
    base.dD = static_cast<uint16_t*>(dD);
    base.C_out = (int)C_out, base.C_in = (int)C_in;
    base.n = n;
    base.mix = seed_mix(seed);
    base.stride = stride, base.P = (int)P, base.Q = (int)Q, base.H = (int)H, base.Wd = (int)Wd;
    base.rows_dO = B * P * Q, base.gather = 1, base.w_taps = R * S;

    int shape;
    if (C_in <= 64) shape = (mode != 0) ? 3 : 2;
    else if (mode != 0 && C_in > 128) shape = 0;
    else shape = 1;
    const int bn = kPwShapes[shape].bn, rows_per = kPwShapes[shape].rows;
    base.ntiles_n = (int)((C_in + bn - 1) / bn);

    // all classes first: nothing is launched unless every one of them fits
    static_assert(kPwMaxClasses >= 16, "stride up to four");
    PwClasses all{};
    PwParams* cls = all.c;
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
    return launch_pw_classes_any(all, ncls, mode, m, shape, rk, stream);
}

}  // namespace sdgp
