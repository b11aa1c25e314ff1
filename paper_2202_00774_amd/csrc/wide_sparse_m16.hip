// Instantiates the eight-wavefront stride-1 kernel for n <= 2 of m = 16 (structured-sparse matrix instruction).
#include "bwd_wide_launch.h"
namespace sdgp {
int launch_wide_sparse_m16(const WideParams& p, int bn, int rk, hipStream_t stream) {
    return launch_wide_rk<2, 16>(p, bn, rk, stream);
}
}  // namespace sdgp
