// Direct-to-LDS tiled checked GEMM: 128x128 workgroup tile, 2x2 wavefronts.
#include "gemm_tile_async.h"

namespace abft {
hipError_t launch_gemm_tile_a128(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    return atile::launch_cfg<128, 128, 2, 2, 4>(check, want_c, want_q, p, s);
}
}  // namespace abft
