// Host side of the row-per-stage kernel: stride-1 filters three taps wide and at most three rows high, with
// enough 512-row tiles to fill the chip; chooses the tile and launches.
#include <algorithm>
#include <climits>

#include "bwd_row.h"

namespace sdgp {

int launch_row_dense(const RowParams& p, int bn, int rows, hipStream_t stream);
int launch_row_sparse_m4(const RowParams& p, int bn, int rows, int rk, hipStream_t stream);
int launch_row_sparse_m8(const RowParams& p, int bn, int rows, int rk, hipStream_t stream);
int launch_row_sparse_m16(const RowParams& p, int bn, int rows, int rk, hipStream_t stream);
int launch_row_masked_m4(const RowParams& p, int bn, int rows, int rk, hipStream_t stream);
int launch_row_masked_m8(const RowParams& p, int bn, int rows, int rk, hipStream_t stream);
int launch_row_masked_m16(const RowParams& p, int bn, int rows, int rk, hipStream_t stream);
int launch_row_masked_m32(const RowParams& p, int bn, int rows, int rk, hipStream_t stream);
int row_lds_bytes(int mode, int bn, int rows, int halo, int npad);

namespace {

// Tile shape for workgroup tiles of `rows` rows: fewest tiles, then least halo, under the LDS budget and the copy
// schedule (16 units per stage).  Returns the number of workgroups, 0 when nothing fits.
int64_t plan_tiles(RowParams& p, int rows, int mode, int bn, int64_t B, int64_t H, int64_t Wd, int R, int S, int64_t P, int64_t Q) {
    const int ntaps = R * S;
    double best = 1e300;
    int bTB = 0, bTH = 0, bTW = 0, bhalo = 0, bnpad = 0;
    for (int TH = 1; TH <= std::min((int)H, rows); ++TH) {
        for (int TW = 1; TW <= std::min((int)Wd, rows / TH); ++TW) {
            const int tb_max = std::max(1, std::min((int)B, rows / (TH * TW)));
            for (int TB = tb_max; TB >= 1; TB = (TB > 1 ? TB / 2 : 0)) {
                // the halo is clipped to the image
                const int halo = TB * (int)std::min<int64_t>(TH + R - 1, P) * (int)std::min<int64_t>(TW + S - 1, Q);
                const int units = (halo + 15) / 16;
                if (units > 16 * R) continue;
                const int npad = TB * (TH + R - 1) * (TW + S - 1);  // the same window with the image borders
                if (row_lds_bytes(mode, bn, rows, halo, npad) > 160 * 1024) continue;
                const double tiles = (double)((B + TB - 1) / TB) * ((H + TH - 1) / TH) * ((Wd + TW - 1) / TW);
                const double cost = tiles * (rows * (double)ntaps + 2.0 * halo + 64.0);
                if (cost < best || (cost == best && TW > bTW)) best = cost, bTB = TB, bTH = TH, bTW = TW, bhalo = halo, bnpad = npad;
            }
        }
    }
    if (bTB == 0) return 0;
    p.TB = bTB, p.TH = bTH, p.TW = bTW;
    p.tiles_h = ((int)H + p.TH - 1) / p.TH;
    p.tiles_w = ((int)Wd + p.TW - 1) / p.TW;
    p.halo_max = bhalo;
    p.npad = bnpad;
    p.ups = (((bhalo + 15) / 16) + R - 1) / R;
    return (int64_t)((B + p.TB - 1) / p.TB) * p.tiles_h * p.tiles_w * p.ntiles_n;
}

}  // namespace

// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.
int bwd_row_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                   int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                   hipStream_t stream) {
    // 0: dense; 2: at most two survivors per aligned quad, the structured-sparse instruction; 1: any other n of m in
    // {4, 8, 16, 32}, the pruned halo stored dense with zeros
    int mode;
    if (n == m) mode = 0;
    else if (n <= 2 && (m == 4 || m == 8 || m == 16)) mode = 2;
    else if (m == 4 || m == 8 || m == 16 || m == 32) mode = 1;
    else return 1;
    if (stride != 1 || S != kRowTaps || R < 1 || R > kRowMaxRows || (C_out % kRowKC) != 0 || (C_in % 8) != 0) return 1;
    if (mode != 0 && (C_out % m) != 0) return 1;
    if (!is_aligned16(dO) || !is_aligned16(W) || !is_aligned16(dD)) return 1;
    const int ntaps = R * S;
    const int64_t P = H + 2 * pad - R + 1, Q = Wd + 2 * pad - S + 1;
    if (P < 1 || Q < 1 || pad < 0) return 1;
    if (B * P * Q >= INT_MAX || B * H * Wd >= INT_MAX || (int64_t)ntaps * C_in >= (1 << 24) ||
        C_out * (int64_t)ntaps * C_in >= (1 << 30) || C_out >= INT_MAX / 2)
        return 1;

    RowParams p{};
    p.dO = static_cast<const uint16_t*>(dO);
    p.W = static_cast<const uint16_t*>(W);
    p.dD = static_cast<uint16_t*>(dD);
    p.B = (int)B, p.P = (int)P, p.Q = (int)Q, p.C_out = (int)C_out, p.C_in = (int)C_in, p.H = (int)H, p.Wd = (int)Wd;
    p.R = R, p.pad = pad;
    p.w_row = ntaps * (int)C_in;
    p.n = n;
    p.mix = seed_mix(seed);

    // 512-row tiles when they fill the chip, else 256-row tiles (twice the workgroups, half the matrix work per stage);
    // 128-column tiles unless they leave a quarter of the CUs without a workgroup: then 64-column tiles, twice as many
    // (measured on the 512 -> 512 layer at 4 x 4: 128 workgroups of 128 columns 57 us, 256 of 64 columns 45 us)
    int bn = (C_in > 64) ? 128 : 64;
    if (mode == 1 && m == 32) bn = 64;  // the 32-key ranker leaves no registers for the 128-column tile's fragments
    int rows = 512;
    int64_t blocks = 0;
    RowParams chosen = p;
    for (;;) {
        RowParams p512 = p, p256 = p;
        p512.ntiles_n = p256.ntiles_n = ((int)C_in + bn - 1) / bn;
        const int64_t n512 = plan_tiles(p512, 512, mode, bn, B, H, Wd, R, S, P, Q);
        const int64_t n256 = plan_tiles(p256, 256, mode, bn, B, H, Wd, R, S, P, Q);
        if (n512 >= 192 || (n512 >= 128 && n256 < 128) || n256 == 0) rows = 512, chosen = p512, blocks = n512;
        else rows = 256, chosen = p256, blocks = n256;
        if (bn == 128 && blocks < 192) {
            bn = 64;
            continue;
        }
        break;
    }
    p = chosen;
    if (blocks == 0 && (B == 0 || H == 0 || Wd == 0)) return SDGP_OK;
    if (blocks < 128 || blocks >= INT_MAX) return 1;  // too few tiles to keep half the chip busy: another kernel takes it
    p.nblocks = (int)blocks;

    if (mode == 0) return launch_row_dense(p, bn, rows, stream);
    if (mode == 1) {
        if (m == 4) return launch_row_masked_m4(p, bn, rows, rk, stream);
        if (m == 8) return launch_row_masked_m8(p, bn, rows, rk, stream);
        if (m == 16) return launch_row_masked_m16(p, bn, rows, rk, stream);
        return launch_row_masked_m32(p, bn, rows, rk, stream);
    }
    if (m == 4) return launch_row_sparse_m4(p, bn, rows, rk, stream);
    if (m == 8) return launch_row_sparse_m8(p, bn, rows, rk, stream);
    return launch_row_sparse_m16(p, bn, rows, rk, stream);
}

}  // namespace sdgp
