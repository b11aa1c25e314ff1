// Instantiates the asynchronous-copy kernel for n <= 2 of m = 16 (structured-sparse matrix instruction).
#include "bwd_conv3_launch.h"
namespace sdgp {
int launch_conv3_sparse_m16(const Conv3Params& p, int bn, int rk, hipStream_t stream) {
    return launch_conv3_rk<2, 16>(p, bn, rk, stream);
}
}  // namespace sdgp
