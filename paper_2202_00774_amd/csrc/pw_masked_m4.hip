// Instantiates the pointwise kernel for any n of m = 4 that the structured-sparse instruction cannot take (n > 2):
// the pruned rows are stored dense with zeros and multiplied by the dense matrix instruction.
#include "bwd_pw_launch.h"
namespace sdgp {
int launch_pw_masked_m4(const PwParams& p, int shape, int rk, hipStream_t stream) {
    return launch_pw_rk<1, 4>(p, shape, rk, stream);
}
int launch_pw_classes_masked_m4(const PwClasses& all, int ncls, int shape, int rk, hipStream_t stream) {
    return launch_pw_classes_rk<1, 4>(all, ncls, shape, rk, stream);
}
}  // namespace sdgp
