// Instantiates the tiled kernel for n <= 2 of m = 8 (compressed halo, structured-sparse matrix instruction).
#include "bwd_tiled_launch.h"
namespace sdgp {
int launch_tiled_sparse_m8(const TiledParams& p, int bn, int rk, hipStream_t stream) {
    return launch_tiled_rk<64, 2, 8>(p, bn, rk, stream);
}
}  // namespace sdgp
