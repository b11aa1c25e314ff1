// Launch helpers for the tiled backward-data kernel; included by the files that instantiate it.
#pragma once

#include "bwd_tiled.h"

namespace sdgp {

constexpr int kLdsPerCu = 160 * 1024;

template <int BN, int KC, int MODE, int M, int RK>
int launch_tiled_one(const TiledParams& p, hipStream_t stream) {
    using L = TiledLayout<BN, KC, MODE>;
    const int lds = L::total(p.halo_max);
    if (lds > kLdsPerCu) return SDGP_ERR_SHAPE;
    auto kern = bwd_tiled<BN, KC, MODE, M, RK>;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsPerCu);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(p.nblocks), dim3(512), lds, stream, p);
    return launch_status();
}

template <int KC, int MODE, int M, int RK>
int launch_tiled_bn(const TiledParams& p, int bn, hipStream_t stream) {
    return bn == 128 ? launch_tiled_one<128, KC, MODE, M, RK>(p, stream) : launch_tiled_one<64, KC, MODE, M, RK>(p, stream);
}

template <int KC, int MODE, int M>
int launch_tiled_rk(const TiledParams& p, int bn, int rk, hipStream_t stream) {
    switch (rk) {
        case kRandom: return launch_tiled_bn<KC, MODE, M, kRandom>(p, bn, stream);
        case kGreedy: return launch_tiled_bn<KC, MODE, M, kGreedy>(p, bn, stream);
        default: return launch_tiled_bn<KC, MODE, M, kAdjusted>(p, bn, stream);
    }
}

// LDS bytes a configuration needs for a halo of `halo` pixels.
template <int KC, int MODE>
int tiled_lds_bytes(int bn, int halo) {
    return bn == 128 ? TiledLayout<128, KC, MODE>::total(halo) : TiledLayout<64, KC, MODE>::total(halo);
}

}  // namespace sdgp
