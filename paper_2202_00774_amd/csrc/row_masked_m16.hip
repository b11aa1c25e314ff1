// Instantiates the row-per-stage kernel for any n of m = 16 that the structured-sparse instruction cannot take (n > 2):
// the pruned halo is stored dense with zeros and multiplied by the dense matrix instruction.
#include "bwd_row_launch.h"
namespace sdgp {
int launch_row_masked_m16(const RowParams& p, int bn, int rows, int rk, hipStream_t stream) {
    return launch_row_rk<1, 16>(p, bn, rows, rk, stream);
}
}  // namespace sdgp
