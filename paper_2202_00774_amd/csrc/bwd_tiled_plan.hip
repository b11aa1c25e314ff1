// Host side of the tiled backward-data kernel: decides whether a problem fits
// it, splits the filter into parity classes, chooses the tile shape and fills
// TiledParams.
#include <algorithm>
#include <climits>

#include "bwd_tiled.h"

namespace sdgp {

int launch_tiled_dense(const TiledParams& p, int bn, hipStream_t stream);
int launch_tiled_sparse_m4(const TiledParams& p, int bn, int rk, hipStream_t stream);
int launch_tiled_sparse_m8(const TiledParams& p, int bn, int rk, hipStream_t stream);
int launch_tiled_sparse_m16(const TiledParams& p, int bn, int rk, hipStream_t stream);
int launch_tiled_masked_m4(const TiledParams& p, int bn, int rk, hipStream_t stream);
int launch_tiled_masked_m8(const TiledParams& p, int bn, int rk, hipStream_t stream);
int launch_tiled_masked_m16(const TiledParams& p, int bn, int rk, hipStream_t stream);
int launch_tiled_masked_m32(const TiledParams& p, int bn, int rk, hipStream_t stream);
int tiled_lds_dense(int bn, int halo);
int tiled_lds_masked(int bn, int halo);
int tiled_lds_sparse(int bn, int halo);

namespace {

// 0 dense (n == m), 1 pruned but stored dense, 2 compressed for the sparse matrix instruction, -1 not taken.
int tiled_mode(int n, int m) {
    if (n == m) return 0;
    if (n <= 2 && (m == 4 || m == 8 || m == 16)) return 2;
    if (m == 4 || m == 8 || m == 16 || m == 32) return 1;
    return -1;
}

int lds_bytes(int mode, int bn, int halo) {
    return mode == 0 ? tiled_lds_dense(bn, halo) : (mode == 1 ? tiled_lds_masked(bn, halo) : tiled_lds_sparse(bn, halo));
}

int floor_div(int a, int b) { return (a >= 0) ? a / b : -((-a + b - 1) / b); }

struct ClassTaps {
    int count = 0;
    int dpmin = 0, dpmax = 0, dqmin = 0, dqmax = 0;
};

}  // namespace

// Returns SDGP_OK after launching, or a positive value when the problem does not fit this kernel
// (the caller then uses the shape-agnostic kernel), or a negative sdgp_status.
int bwd_tiled_launch(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                     int64_t C_out, int R, int S, int stride, int pad, int n, int m, int rk, uint64_t seed,
                     hipStream_t stream) {
    const int mode = tiled_mode(n, m);
    if (mode < 0) return 1;
    if ((C_out % 8) != 0 || (C_in % 8) != 0 || stride > 2 || R * S > kMaxTaps) return 1;
    if (!is_aligned16(dO) || !is_aligned16(W)) return 1;
    int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    // A 1x1 stride-1 layer (and a linear layer) has no spatial structure: treat it as one long row of pixels.
    if (R == 1 && S == 1 && stride == 1 && pad == 0) {
        Wd = B * H * Wd;
        Q = Wd;
        B = 1, H = 1, P = 1;
    }
    if (B * P * Q >= INT_MAX || B * H * Wd >= INT_MAX || (int64_t)R * S * C_in >= INT_MAX || C_out >= INT_MAX / 2)
        return 1;
    // the random ranker hashes a 16-channel item with one high word of the flat element index: items start at multiples
    // of 16 elements, or the tensor stays below 2^32 elements
    if ((C_out % 16) != 0 && B * P * Q * C_out >= ((int64_t)1 << 32)) return 1;

    TiledParams p{};
    p.dO = static_cast<const uint16_t*>(dO);
    p.W = static_cast<const uint16_t*>(W);
    p.dD = static_cast<uint16_t*>(dD);
    p.B = (int)B, p.P = (int)P, p.Q = (int)Q, p.C_out = (int)C_out, p.C_in = (int)C_in, p.H = (int)H, p.Wd = (int)Wd;
    p.stride = stride;
    p.w_row = R * S * (int)C_in;
    p.n = n;
    p.mix = seed_mix(seed);

    // ---- parity classes and their taps
    p.nclass = stride * stride;
    ClassTaps ct[kMaxClasses];
    int ntaps = 0;
    for (int ph = 0; ph < stride; ++ph) {
        for (int pw = 0; pw < stride; ++pw) {
            const int c = ph * stride + pw;
            TileClass& cl = p.cls[c];
            cl.ph = ph, cl.pw = pw;
            cl.HH = ((int)H - ph + stride - 1) / stride;
            cl.WW = ((int)Wd - pw + stride - 1) / stride;
            cl.tap_begin = ntaps;
            for (int r = 0; r < R; ++r) {
                const int ar = ph + pad - r;
                if (((ar % stride) + stride) % stride != 0) continue;
                for (int s = 0; s < S; ++s) {
                    const int as = pw + pad - s;
                    if (((as % stride) + stride) % stride != 0) continue;
                    TapEntry& t = p.taps[ntaps++];
                    t.dp = floor_div(ar, stride), t.dq = floor_div(as, stride);
                    t.woff = (r * S + s) * (int)C_in;
                    ClassTaps& x = ct[c];
                    if (x.count == 0) x.dpmin = x.dpmax = t.dp, x.dqmin = x.dqmax = t.dq;
                    x.dpmin = std::min(x.dpmin, t.dp), x.dpmax = std::max(x.dpmax, t.dp);
                    x.dqmin = std::min(x.dqmin, t.dq), x.dqmax = std::max(x.dqmax, t.dq);
                    ++x.count;
                }
            }
            cl.tap_count = ct[c].count;
            cl.dpmin = ct[c].dpmin, cl.dqmin = ct[c].dqmin;
        }
    }

    const int bn = (C_in > 64) ? 128 : 64;
    p.ntiles_n = ((int)C_in + bn - 1) / bn;

    // ---- tile shape: minimise (matrix work + halo traffic) summed over classes, under the LDS budget
    // (one workgroup of eight wavefronts per CU).
    const int items_per_pix = (mode == 1 && m == 32) ? 2 : 4;
    double best = 1e300;
    int bTB = 0, bTH = 0, bTW = 0;
    const int maxH = std::max(p.cls[0].HH, 1), maxW = std::max(p.cls[0].WW, 1);
    for (int TH = 1; TH <= std::min(maxH, kTileRows); ++TH) {
        for (int TW = 1; TW <= std::min(maxW, kTileRows / TH); ++TW) {
            const int tb_max = std::max(1, std::min((int)B, kTileRows / (TH * TW)));
            // whole images per tile only pay off for small images; try the largest count and its halvings
            for (int TB = tb_max; TB >= 1; TB = (TB > 1 ? TB / 2 : 0)) {
                double cost = 0;
                int halo_max = 0;
                for (int c = 0; c < p.nclass; ++c) {
                    const TileClass& cl = p.cls[c];
                    if (cl.HH <= 0 || cl.WW <= 0) continue;
                    const double tiles = (double)((B + TB - 1) / TB) * ((cl.HH + TH - 1) / TH) * ((cl.WW + TW - 1) / TW);
                    const int halo = TB * (TH + ct[c].dpmax - ct[c].dpmin) * (TW + ct[c].dqmax - ct[c].dqmin);
                    halo_max = std::max(halo_max, halo);
                    cost += tiles * (kTileRows * (double)ct[c].count * p.ntiles_n + 3.0 * halo * p.ntiles_n + 64.0);
                }
                const int lds = lds_bytes(mode, bn, halo_max);
                if (lds > 160 * 1024) continue;
                if (halo_max * items_per_pix > 256 * kMaxHaloItems) continue;  // a producer lane holds at most that many
                if (cost < best || (cost == best && TW > bTW)) best = cost, bTB = TB, bTH = TH, bTW = TW;
            }
        }
    }
    if (bTB == 0) return 1;
    p.TB = bTB, p.TH = bTH, p.TW = bTW;

    int tiles = 0;
    p.halo_max = 1;
    for (int c = 0; c < p.nclass; ++c) {
        TileClass& cl = p.cls[c];
        cl.tiles_h = std::max(0, (cl.HH + p.TH - 1) / p.TH);
        cl.tiles_w = std::max(0, (cl.WW + p.TW - 1) / p.TW);
        cl.HTH = p.TH + ct[c].dpmax - ct[c].dpmin;
        cl.HTW = p.TW + ct[c].dqmax - ct[c].dqmin;
        cl.tile_base = tiles;
        const int64_t t = (int64_t)((B + p.TB - 1) / p.TB) * cl.tiles_h * cl.tiles_w;
        if (tiles + t >= INT_MAX / 8) return 1;
        tiles += (int)t;
        p.halo_max = std::max(p.halo_max, p.TB * cl.HTH * cl.HTW);
        if (cl.tiles_h == 0 || cl.tiles_w == 0) cl.tiles_h = cl.tiles_w = 1;  // empty class: owns no tile, avoid /0
    }
    // Classes that own no tile must not capture tile ids: give them an unreachable base.
    for (int c = 0; c < p.nclass; ++c)
        if (p.cls[c].HH <= 0 || p.cls[c].WW <= 0) p.cls[c].tile_base = INT_MAX;
    if ((int64_t)tiles * p.ntiles_n >= INT_MAX) return 1;
    p.nblocks = tiles * p.ntiles_n;
    if (p.nblocks == 0) return SDGP_OK;

    switch (mode) {
        case 0: return launch_tiled_dense(p, bn, stream);
        case 2:
            if (m == 4) return launch_tiled_sparse_m4(p, bn, rk, stream);
            if (m == 8) return launch_tiled_sparse_m8(p, bn, rk, stream);
            return launch_tiled_sparse_m16(p, bn, rk, stream);
        default:
            if (m == 4) return launch_tiled_masked_m4(p, bn, rk, stream);
            if (m == 8) return launch_tiled_masked_m8(p, bn, rk, stream);
            if (m == 16) return launch_tiled_masked_m16(p, bn, rk, stream);
            return launch_tiled_masked_m32(p, bn, rk, stream);
    }
}

}  // namespace sdgp
