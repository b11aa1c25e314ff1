// Instantiates the row-per-stage kernel for any n of m = 32 (a group is the whole 32-channel chunk of a pixel):
// the pruned halo is stored dense with zeros and multiplied by the dense matrix instruction.
#include "bwd_row_launch.h"
namespace sdgp {
int launch_row_masked_m32(const RowParams& p, int bn, int rows, int rk, hipStream_t stream) {
    return launch_row_rk<1, 32>(p, bn, rows, rk, stream);
}
}  // namespace sdgp
