// Launch helpers for the row-per-stage kernel; included by the files that instantiate it.
#pragma once

#include "bwd_row.h"

namespace sdgp {

template <int BN, int MODE, int M, int RK, int ROWS>
int launch_row_one(const RowParams& p, hipStream_t stream) {
    using L = RowLayout<BN, MODE, ROWS>;
    const int lds = L::total(p.halo_max, p.npad);
    if (lds > 160 * 1024) return SDGP_ERR_SHAPE;
    auto kern = bwd_row<BN, MODE, M, RK, ROWS>;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return SDGP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(p.nblocks), dim3(512), lds, stream, p);
    return launch_status();
}

template <int MODE, int M, int RK>
int launch_row_bn(const RowParams& p, int bn, int rows, hipStream_t stream) {
    if (rows == 512) return bn == 128 ? launch_row_one<128, MODE, M, RK, 512>(p, stream) : launch_row_one<64, MODE, M, RK, 512>(p, stream);
    return bn == 128 ? launch_row_one<128, MODE, M, RK, 256>(p, stream) : launch_row_one<64, MODE, M, RK, 256>(p, stream);
}

template <int MODE, int M>
int launch_row_rk(const RowParams& p, int bn, int rows, int rk, hipStream_t stream) {
    switch (rk) {
        case kRandom: return launch_row_bn<MODE, M, kRandom>(p, bn, rows, stream);
        case kGreedy: return launch_row_bn<MODE, M, kGreedy>(p, bn, rows, stream);
        default: return launch_row_bn<MODE, M, kAdjusted>(p, bn, rows, stream);
    }
}

}  // namespace sdgp
