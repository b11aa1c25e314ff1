// Instantiates the tiled kernel without pruning (n == m): the dense backward-data baseline.
#include "bwd_tiled_launch.h"
namespace sdgp {
int launch_tiled_dense(const TiledParams& p, int bn, hipStream_t stream) {
    return launch_tiled_bn<64, 0, 4, kGreedy>(p, bn, stream);
}
int tiled_lds_dense(int bn, int halo) { return tiled_lds_bytes<64, 0>(bn, halo); }
int tiled_lds_masked(int bn, int halo) { return tiled_lds_bytes<64, 1>(bn, halo); }
int tiled_lds_sparse(int bn, int halo) { return tiled_lds_bytes<64, 2>(bn, halo); }
}  // namespace sdgp
