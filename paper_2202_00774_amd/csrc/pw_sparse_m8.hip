// Instantiates the pointwise kernel for n <= 2 of m = 8 (structured-sparse matrix instruction).
#include "bwd_pw_launch.h"
namespace sdgp {
int launch_pw_sparse_m8(const PwParams& p, int shape, int rk, hipStream_t stream) {
    return launch_pw_rk<2, 8>(p, shape, rk, stream);
}
int launch_pw_classes_sparse_m8(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream) {
    return launch_pw_classes_rk<2, 8>(all, ncls, shape, rk, stream);
}
}  // namespace sdgp
