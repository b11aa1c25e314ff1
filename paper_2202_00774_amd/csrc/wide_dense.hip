// Instantiates the eight-wavefront stride-1 kernel without pruning (n == m): the dense baseline of the 3x3 layers.
#include "bwd_wide_launch.h"
namespace sdgp {
int launch_wide_dense(const WideParams& p, int bn, hipStream_t stream) {
    return launch_wide_bn<0, 4, kGreedy>(p, bn, stream);
}
int wide_lds_bytes(int mode, int bn, int halo) {
    if (mode == 0) return bn == 128 ? WideLayout<128, 0>::total(halo) : WideLayout<64, 0>::total(halo);
    return bn == 128 ? WideLayout<128, 2>::total(halo) : WideLayout<64, 2>::total(halo);
}
int wide_halo_units_per_stage(int mode, int bn) {
    if (mode == 0) return bn == 128 ? WideLayout<128, 0>::kHU : WideLayout<64, 0>::kHU;
    return bn == 128 ? WideLayout<128, 2>::kHU : WideLayout<64, 2>::kHU;
}
}  // namespace sdgp
