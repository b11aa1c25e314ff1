// Instantiates the eight-wavefront stride-1 kernel for n <= 2 of m = 8 (structured-sparse matrix instruction).
#include "bwd_wide_launch.h"
namespace sdgp {
int launch_wide_sparse_m8(const WideParams& p, int bn, int rk, hipStream_t stream) {
    return launch_wide_rk<2, 8>(p, bn, rk, stream);
}
}  // namespace sdgp
