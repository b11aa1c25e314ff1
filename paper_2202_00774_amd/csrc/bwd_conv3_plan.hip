// Host side of the asynchronous-copy kernel: takes stride-1 filters with at least four taps whose
// channel counts fit (C_out a multiple of 64, C_in a multiple of 8), chooses the tile and launches.
#include <algorithm>
#include <climits>

#include "bwd_conv3.h"

namespace sdgp {

int launch_conv3_dense(const Conv3Params& p, int bn, hipStream_t stream);
int launch_conv3_sparse_m4(const Conv3Params& p, int bn, int rk, hipStream_t stream);
int launch_conv3_sparse_m8(const Conv3Params& p, int bn, int rk, hipStream_t stream);
int launch_conv3_sparse_m16(const Conv3Params& p, int bn, int rk, hipStream_t stream);
int conv3_lds_bytes(int mode, int bn, int halo);

// SDGP_OK after launching, a positive value when the problem does not fit, or a negative sdgp_status.
int bwd_conv3_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                     int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                     hipStream_t stream) {
    int mode;
    if (n == m) mode = 0;
    else if (n <= 2 && (m == 4 || m == 8 || m == 16)) mode = 2;
    else return 1;
    const int ntaps = R * S;
    if (stride != 1 || ntaps < 4 || ntaps > kMaxTaps || (C_out % kC3KC) != 0 || C_out > kC3MaxCout || (C_in % 8) != 0) return 1;
    if (!is_aligned16(dO) || !is_aligned16(W)) return 1;
    const int64_t P = H + 2 * pad - R + 1, Q = Wd + 2 * pad - S + 1;
    if (B * P * Q >= INT_MAX || B * H * Wd >= INT_MAX || (int64_t)ntaps * C_in >= (1 << 24) || C_out >= INT_MAX / 2) return 1;

    Conv3Params p{};
    p.dO = static_cast<const uint16_t*>(dO);
    p.W = static_cast<const uint16_t*>(W);
    p.dD = static_cast<uint16_t*>(dD);
    p.B = (int)B, p.P = (int)P, p.Q = (int)Q, p.C_out = (int)C_out, p.C_in = (int)C_in, p.H = (int)H, p.Wd = (int)Wd;
    p.w_row = ntaps * (int)C_in;
    p.n = n;
    p.mix = seed_mix(seed);
    p.ntaps = ntaps;
    // dD[h, w] gathers dO[h + pad - r, w + pad - s]
    for (int r = 0; r < R; ++r)
        for (int s = 0; s < S; ++s) {
            TapEntry& t = p.taps[r * S + s];
            t.dp = pad - r, t.dq = pad - s, t.woff = (r * S + s) * (int)C_in;
        }
    p.dpmin = pad - (R - 1), p.dqmin = pad - (S - 1);

    const int bn = (C_in > 64) ? 128 : 64;
    p.ntiles_n = ((int)C_in + bn - 1) / bn;
    const int nb = (mode == 2) ? ntaps - 1 : ntaps - 3;  // stages per chunk that carry halo copies

    double best = 1e300;
    int bTB = 0, bTH = 0, bTW = 0;
    for (int TH = 1; TH <= std::min((int)H, kTileRows); ++TH) {
        for (int TW = 1; TW <= std::min((int)Wd, kTileRows / TH); ++TW) {
            const int tb_max = std::max(1, std::min((int)B, kTileRows / (TH * TW)));
            for (int TB = tb_max; TB >= 1; TB = (TB > 1 ? TB / 2 : 0)) {
                const int halo = TB * (TH + R - 1) * (TW + S - 1);
                const int units = (halo + 7) / 8;
                if (units > kC3UnitsPerStep * nb) continue;
                if (conv3_lds_bytes(mode, bn, halo) > 160 * 1024) continue;
                const double tiles = (double)((B + TB - 1) / TB) * ((H + TH - 1) / TH) * ((Wd + TW - 1) / TW);
                const double cost = tiles * (kTileRows * (double)ntaps + 3.0 * halo + 64.0);
                if (cost < best || (cost == best && TW > bTW)) best = cost, bTB = TB, bTH = TH, bTW = TW;
            }
        }
    }
    if (bTB == 0) return 1;
    p.TB = bTB, p.TH = bTH, p.TW = bTW;
    p.tiles_h = ((int)H + p.TH - 1) / p.TH;
    p.tiles_w = ((int)Wd + p.TW - 1) / p.TW;
    p.HTH = p.TH + R - 1, p.HTW = p.TW + S - 1;
    p.nhalo = p.TB * p.HTH * p.HTW;
    p.nunits = (p.nhalo + 7) / 8;
    const int64_t tiles = (int64_t)((B + p.TB - 1) / p.TB) * p.tiles_h * p.tiles_w;
    if (tiles * p.ntiles_n >= INT_MAX) return 1;
    p.nblocks = (int)tiles * p.ntiles_n;
    if (p.nblocks == 0) return SDGP_OK;

    if (mode == 0) return launch_conv3_dense(p, bn, stream);
    if (m == 4) return launch_conv3_sparse_m4(p, bn, rk, stream);
    if (m == 8) return launch_conv3_sparse_m8(p, bn, rk, stream);
    return launch_conv3_sparse_m16(p, bn, rk, stream);
}

}  // namespace sdgp
