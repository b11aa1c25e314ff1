// Instantiates the row-per-stage kernel without pruning (n == m): the dense baseline of the 3x3 layers.
#include "bwd_row_launch.h"
namespace sdgp {
int launch_row_dense(const RowParams& p, int bn, int rows, hipStream_t stream) {
    return launch_row_bn<0, 4, kGreedy>(p, bn, rows, stream);
}
int row_lds_bytes(int mode, int bn, int rows, int halo) {
    if (rows == 512) {
        if (mode == 0) return bn == 128 ? RowLayout<128, 0, 512>::total(halo) : RowLayout<64, 0, 512>::total(halo);
        return bn == 128 ? RowLayout<128, 2, 512>::total(halo) : RowLayout<64, 2, 512>::total(halo);
    }
    if (mode == 0) return bn == 128 ? RowLayout<128, 0, 256>::total(halo) : RowLayout<64, 0, 256>::total(halo);
    return bn == 128 ? RowLayout<128, 2, 256>::total(halo) : RowLayout<64, 2, 256>::total(halo);
}
}  // namespace sdgp
