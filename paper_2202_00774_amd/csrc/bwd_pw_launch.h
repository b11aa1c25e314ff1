// Launch helpers for the pointwise (1x1 / linear) kernel; included by the files that instantiate it.
#pragma once

#include "bwd_pw.h"

namespace sdgp {

template <int BN, int MODE, int M, int RK, int ROWS>
int launch_pw_one(const PwParams& p, hipStream_t stream) {
    using L = PwLayout<BN, MODE, ROWS>;
    auto kern = bwd_pw<BN, MODE, M, RK, ROWS>;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(p.nblocks), dim3(512), L::total(), stream, p);
    return launch_status();
}

// shape: 0 = 256 rows x 256 columns, 1 = 512 x 128, 2 = 256 x 128, 3 = 512 x 64
template <int MODE, int M, int RK>
int launch_pw_shape(const PwParams& p, int shape, hipStream_t stream) {
    switch (shape) {
        case 0: return launch_pw_one<256, MODE, M, RK, 256>(p, stream);
        case 1: return launch_pw_one<128, MODE, M, RK, 512>(p, stream);
        case 2: return launch_pw_one<128, MODE, M, RK, 256>(p, stream);
        default: return launch_pw_one<64, MODE, M, RK, 512>(p, stream);
    }
}

template <int MODE, int M>
int launch_pw_rk(const PwParams& p, int shape, int rk, hipStream_t stream) {
    switch (rk) {
        case kRandom: return launch_pw_shape<MODE, M, kRandom>(p, shape, stream);
        case kGreedy: return launch_pw_shape<MODE, M, kGreedy>(p, shape, stream);
        default: return launch_pw_shape<MODE, M, kAdjusted>(p, shape, stream);
    }
}

}  // namespace sdgp
