// Instantiates the pointwise kernel for a gradient that arrives ranked and compressed (MODE 3; csrc/compress.hip).
#include "bwd_pw_launch.h"
namespace sdgp {
int launch_pw_pre(const PwParams& p, int shape, hipStream_t stream) {
    return launch_pw_shape<3, 4, kGreedy>(p, shape, stream);
}
int launch_pw_classes_pre(const PwClasses& all, int ncls, int shape, hipStream_t stream) {
    return launch_pw_classes_shape<3, 4, kGreedy>(all, ncls, shape, stream);
}
}  // namespace sdgp
