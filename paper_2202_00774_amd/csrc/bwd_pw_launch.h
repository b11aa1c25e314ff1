// Launch helpers for the pointwise (1x1 / linear) kernel; included by the files that instantiate it.
#pragma once

#include "bwd_pw.h"

namespace sdgp {

template <int BN, int MODE, int M, int RK, int ROWS, int NW, bool GATHER>
int launch_pw_one(const PwParams& p, hipStream_t stream) {
    using L = PwLayout<BN, MODE, ROWS>;
    auto kern = bwd_pw<BN, MODE, M, RK, ROWS, NW, GATHER>;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(p.nblocks), dim3(NW * 64), L::total(), stream, p);
    return launch_status();
}

// tile shapes: columns, rows, wavefronts
struct PwShape {
    int bn, rows, waves;
};
constexpr PwShape kPwShapes[] = {{256, 128, 4}, {128, 128, 4}, {64, 256, 4}};
constexpr int kPwNumShapes = sizeof(kPwShapes) / sizeof(kPwShapes[0]);

template <int MODE, int M, int RK>
int launch_pw_shape(const PwParams& p, int shape, hipStream_t stream) {
    switch (shape) {
#define SDGP_PW_CASE(i) \
    case i:                                                                                                          \
        return p.gather ? launch_pw_one<kPwShapes[i].bn, MODE, M, RK, kPwShapes[i].rows, kPwShapes[i].waves, true>(p, stream)  \
                        : launch_pw_one<kPwShapes[i].bn, MODE, M, RK, kPwShapes[i].rows, kPwShapes[i].waves, false>(p, stream);
        SDGP_PW_CASE(0)
        SDGP_PW_CASE(1)
        SDGP_PW_CASE(2)
#undef SDGP_PW_CASE
        default: return SDGP_ERR_SHAPE;
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
