// Instantiates the row-per-stage kernel without pruning (n == m): the dense baseline of the 3x3 layers.
#include "bwd_row_launch.h"
namespace sdgp {
int launch_row_dense(const RowParams& p, int bn, hipStream_t stream) {
    return launch_row_bn<0, 4, kGreedy>(p, bn, stream);
}
int row_lds_bytes(int mode, int bn, int halo) {
    if (mode == 0) return bn == 128 ? RowLayout<128, 0>::total(halo) : RowLayout<64, 0>::total(halo);
    return bn == 128 ? RowLayout<128, 2>::total(halo) : RowLayout<64, 2>::total(halo);
}
}  // namespace sdgp
