// Host side of the pointwise kernel: 1x1 convolutions without padding (any stride) and linear layers whose channel
// counts fit (C_out a multiple of 32, C_in a multiple of 8); chooses the tile shape and launches.
#include <climits>
#include <cstdlib>

#include "bwd_pw_launch.h"

namespace sdgp {

int launch_pw_dense(const PwParams& p, int shape, hipStream_t stream);
int launch_pw_sparse_m4(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_sparse_m8(const PwParams& p, int shape, int rk, hipStream_t stream);
int launch_pw_sparse_m16(const PwParams& p, int shape, int rk, hipStream_t stream);

// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.
int bwd_pw_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                  int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed, hipStream_t stream) {
    int mode;
    if (n == m) mode = 0;
    else if (n <= 2 && (m == 4 || m == 8 || m == 16)) mode = 2;
    else return 1;
    if (R != 1 || S != 1 || stride < 1 || stride > 255 || pad != 0 || (C_out % kPwKC) != 0 || (C_in % 8) != 0) return 1;
    if (mode == 2 && (C_out % m) != 0) return 1;
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
    p.mix = seed_mix(seed);

    // tile shape.  Workgroups of four wavefronts, two to a CU, so that one's loads and stores overlap the other's
    // arithmetic.  Pruning: all of C_in (up to 256 columns) in one workgroup, so every gradient row is ranked once;
    // dense: 128 x 128 tiles measured fastest (column tiles of one row tile run side by side on one XCD and find
    // the gradient rows in its L2).
    auto blocks_of = [&](int rows_per, int bn) { return ((rows + rows_per - 1) / rows_per) * ((C_in + bn - 1) / bn); };
    int shape;
    if (C_in <= 64) shape = 2;
    else if (mode == 2 && C_in > 128) shape = 0;
    else shape = 1;
#ifdef SDGP_TRACE
    if (const char* e = getenv("SDGP_PW_SHAPE")) {
        const int v = atoi(e);
        if (v >= 0 && v < kPwNumShapes) shape = v;
    }
#endif
    const int bn = kPwShapes[shape].bn, rows_per = kPwShapes[shape].rows;
    const int64_t blocks = blocks_of(rows_per, bn);
    if (blocks < 64 || blocks >= INT_MAX) return 1;  // too small to be worth a matrix-core launch of this shape
    p.ntiles_n = (int)((C_in + bn - 1) / bn);
    p.nblocks = (int)blocks;

    if (mode == 0) return launch_pw_dense(p, shape, stream);
    if (m == 4) return launch_pw_sparse_m4(p, shape, rk, stream);
    if (m == 8) return launch_pw_sparse_m8(p, shape, rk, stream);
    return launch_pw_sparse_m16(p, shape, rk, stream);
}

}  // namespace sdgp
