// Direct-to-LDS tiled checked GEMM: 256x256 workgroup tile, 4x2 wavefronts.
#include "gemm_tile_async.h"

namespace abft {
hipError_t launch_gemm_tile_a256w42(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    return atile::launch_cfg<256, 256, 4, 2, 2>(check, want_c, want_q, p, s);
}
}  // namespace abft
