// Instantiates the row-per-stage kernel for n <= 2 of m = 4 (structured-sparse matrix instruction).
#include "bwd_row_launch.h"
namespace sdgp {
int launch_row_sparse_m4(const RowParams& p, int bn, int rows, int rk, hipStream_t stream) {
    return launch_row_rk<2, 4>(p, bn, rows, rk, stream);
}
}  // namespace sdgp
