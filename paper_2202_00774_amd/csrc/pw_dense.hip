// Instantiates the pointwise kernel without pruning (n == m): the dense baseline of the 1x1 and linear layers.
#include "bwd_pw_launch.h"
namespace sdgp {
int launch_pw_dense(const PwParams& p, int shape, hipStream_t stream) {
    return launch_pw_shape<0, 4, kGreedy>(p, shape, stream);
}
int launch_pw_classes_dense(const PwClasses& all, int ncls, int shape, hipStream_t stream) {
    return launch_pw_classes_shape<0, 4, kGreedy>(all, ncls, shape, stream);
}
}  // namespace sdgp
