// Instantiates the asynchronous-copy kernel without pruning (n == m): the dense baseline of the 3x3 layers.
#include "bwd_conv3_launch.h"
namespace sdgp {
int launch_conv3_dense(const Conv3Params& p, int bn, hipStream_t stream) {
    return launch_conv3_bn<0, 4, kGreedy>(p, bn, stream);
}
int conv3_lds_bytes(int mode, int bn, int halo) {
    if (mode == 0) return bn == 128 ? Conv3Layout<128, 0>::total(halo) : Conv3Layout<64, 0>::total(halo);
    return bn == 128 ? Conv3Layout<128, 2>::total(halo) : Conv3Layout<64, 2>::total(halo);
}
}  // namespace sdgp
