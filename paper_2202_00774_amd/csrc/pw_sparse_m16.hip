// Instantiates the pointwise kernel for n <= 2 of m = 16 (structured-sparse matrix instruction).
#include "bwd_pw_launch.h"
namespace sdgp {
int launch_pw_sparse_m16(const PwParams& p, int shape, int rk, hipStream_t stream) {
    return launch_pw_rk<2, 16>(p, shape, rk, stream);
}
int launch_pw_classes_sparse_m16(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream) {
    return launch_pw_classes_rk<2, 16>(all, ncls, shape, rk, stream);
}
}  // namespace sdgp
