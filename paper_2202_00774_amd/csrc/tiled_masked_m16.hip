// Instantiates the tiled kernel for 2 < n < m = 16 (pruned halo stored dense, dense matrix instruction).
#include "bwd_tiled_launch.h"
namespace sdgp {
int launch_tiled_masked_m16(const TiledParams& p, int bn, int rk, hipStream_t stream) {
    return launch_tiled_rk<64, 1, 16>(p, bn, rk, stream);
}
}  // namespace sdgp
