// Direct-to-LDS tiled checked GEMM: 64x64 workgroup tile, K split between two groups of 2x2 wavefronts
// (32x32 each), a ring of four stages per group.
#include "gemm_tile_async.h"

namespace abft {
hipError_t launch_gemm_tile_a64k2(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    return atile::launch_cfg<64, 64, 2, 2, 4, 2>(check, want_c, want_q, p, s);
}
}  // namespace abft
