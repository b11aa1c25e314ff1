// Instantiates the row-per-stage kernel without pruning (n == m): the dense baseline of the 3x3 layers.
#include "bwd_row_launch.h"
namespace sdgp {
int launch_row_dense(const RowParams& p, int bn, int rows, hipStream_t stream) {
    return launch_row_bn<0, 4, kGreedy>(p, bn, rows, stream);
}
int row_lds_bytes(int mode, int bn, int rows, int halo, int npad) {
#define SDGP_ROW_LDS(MODE)                                                                                       \
    (rows == 512 ? (bn == 128 ? RowLayout<128, MODE, 512>::total(halo, npad) : RowLayout<64, MODE, 512>::total(halo, npad)) \
                 : (bn == 128 ? RowLayout<128, MODE, 256>::total(halo, npad) : RowLayout<64, MODE, 256>::total(halo, npad)))
    if (mode == 0) return SDGP_ROW_LDS(0);
    if (mode == 1) return SDGP_ROW_LDS(1);
    return SDGP_ROW_LDS(2);
#undef SDGP_ROW_LDS
}
}  // namespace sdgp
