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

template <int BN, int MODE, int M, int RK, int ROWS, int NW>
int launch_pw_classes_one(const PwClasses& all, int ncls, hipStream_t stream) {
    using L = PwLayout<BN, MODE, ROWS>;
    auto kern = bwd_pw_classes<BN, MODE, M, RK, ROWS, NW>;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    int widest = 0;
    for (int i = 0; i < ncls; ++i) widest = all.c[i].nblocks > widest ? all.c[i].nblocks : widest;
    hipLaunchKernelGGL(kern, dim3(widest, ncls), dim3(NW * 64), L::total(), stream, all);
    return launch_status();
}

// tile shapes: columns, rows, wavefronts
struct PwShape {
    int bn, rows, waves;
};
constexpr PwShape kPwShapes[] = {{256, 128, 4}, {128, 128, 4}, {64, 256, 4}, {64, 128, 4}};
constexpr int kPwNumShapes = sizeof(kPwShapes) / sizeof(kPwShapes[0]);

template <int MODE, int M, int RK>
int launch_pw_shape(const PwParams& p, int shape, hipStream_t stream) {
    switch (shape) {
#define SDGP_PW_CASE(i) \
    case i:                                                                                                          \
        return launch_pw_one<kPwShapes[i].bn, MODE, M, RK, kPwShapes[i].rows, kPwShapes[i].waves, false>(p, stream);
        SDGP_PW_CASE(0)
        SDGP_PW_CASE(1)
        SDGP_PW_CASE(2)
        SDGP_PW_CASE(3)
#undef SDGP_PW_CASE
        default: return SDGP_ERR_SHAPE;
    }
}

template <int MODE, int M, int RK>
int launch_pw_classes_shape(const PwClasses& all, int ncls, int shape, hipStream_t stream) {
    switch (shape) {
#define SDGP_PW_CASE(i) \
    case i: return launch_pw_classes_one<kPwShapes[i].bn, MODE, M, RK, kPwShapes[i].rows, kPwShapes[i].waves>(all, ncls, stream);
        SDGP_PW_CASE(0)
        SDGP_PW_CASE(1)
        SDGP_PW_CASE(2)
        SDGP_PW_CASE(3)
#undef SDGP_PW_CASE
        default: return SDGP_ERR_SHAPE;
    }
}

template <int MODE, int M>
int launch_pw_classes_rk(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream) {
    switch (rk) {
        case kRandom: return launch_pw_classes_shape<MODE, M, kRandom>(all, ncls, shape, stream);
        case kGreedy: return launch_pw_classes_shape<MODE, M, kGreedy>(all, ncls, shape, stream);
        default: return launch_pw_classes_shape<MODE, M, kAdjusted>(all, ncls, shape, stream);
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
