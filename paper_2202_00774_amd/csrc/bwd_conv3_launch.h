// Launch helpers for the asynchronous-copy kernel; included by the files that instantiate it.
#pragma once

#include "bwd_conv3.h"

namespace sdgp {

template <int BN, int MODE, int M, int RK>
int launch_conv3_one(const Conv3Params& p, hipStream_t stream) {
    using L = Conv3Layout<BN, MODE>;
    const int lds = L::total(p.nhalo);
    if (lds > 160 * 1024) return SDGP_ERR_SHAPE;
    auto kern = bwd_conv3<BN, MODE, M, RK>;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(p.nblocks), dim3(conv3_threads(MODE)), lds, stream, p);
    return launch_status();
}

template <int MODE, int M, int RK>
int launch_conv3_bn(const Conv3Params& p, int bn, hipStream_t stream) {
    return bn == 128 ? launch_conv3_one<128, MODE, M, RK>(p, stream) : launch_conv3_one<64, MODE, M, RK>(p, stream);
}

template <int MODE, int M>
int launch_conv3_rk(const Conv3Params& p, int bn, int rk, hipStream_t stream) {
    switch (rk) {
        case kRandom: return launch_conv3_bn<MODE, M, kRandom>(p, bn, stream);
        case kGreedy: return launch_conv3_bn<MODE, M, kGreedy>(p, bn, stream);
        default: return launch_conv3_bn<MODE, M, kAdjusted>(p, bn, stream);
    }
}

}  // namespace sdgp
