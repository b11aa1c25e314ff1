// Host side of the pointwise kernel: 1x1 stride-1 convolutions without padding and linear layers whose channel
// counts fit (C_out a multiple of 32, C_in a multiple of 8); chooses the tile shape and launches.
#include <climits>

#include "bwd_pw.h"

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
    if (R != 1 || S != 1 || stride != 1 || pad != 0 || (C_out % kPwKC) != 0 || (C_in % 8) != 0) return 1;
    if (mode == 2 && (C_out % m) != 0) return 1;
    if (!is_aligned16(dO) || !is_aligned16(W) || !is_aligned16(dD)) return 1;
    const int64_t rows = B * H * Wd;
    if (rows < 1 || C_out < kPwKC || C_in < 8 || C_out >= (1 << 24) || C_in >= (1 << 24)) return 1;

    PwParams p{};
    p.dO = static_cast<const uint16_t*>(dO);
    p.W = static_cast<const uint16_t*>(W);
    p.dD = static_cast<uint16_t*>(dD);
    p.rows = rows, p.C_out = (int)C_out, p.C_in = (int)C_in;
    p.n = n;
    p.mix = seed_mix(seed);

    // tile shape: all of C_in in one workgroup when it fits (the gradient is then read from HBM once); the larger
    // row tile when it still gives every CU a workgroup
    auto blocks_of = [&](int rows_per, int bn) { return ((rows + rows_per - 1) / rows_per) * ((C_in + bn - 1) / bn); };
    int shape, bn, rows_per;
    if (C_in > 128) {
        if (blocks_of(256, 256) >= 256) shape = 0, bn = 256, rows_per = 256;
        else shape = 2, bn = 128, rows_per = 256;
    } else if (C_in > 64) {
        if (blocks_of(512, 128) >= 256) shape = 1, bn = 128, rows_per = 512;
        else shape = 2, bn = 128, rows_per = 256;
    } else {
        shape = 3, bn = 64, rows_per = 512;
    }
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
