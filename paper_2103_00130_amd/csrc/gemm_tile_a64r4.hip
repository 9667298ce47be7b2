// Direct-to-LDS tiled checked GEMM: 64x64 workgroup tile, 2x2 wavefronts, a ring of four stages (grids of at
// most one workgroup per compute unit with a short K: the whole ring is in flight before the first k-step).
#include "gemm_tile_async.h"

namespace abft {
hipError_t launch_gemm_tile_a64r4(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    return atile::launch_cfg<64, 64, 2, 2, 4>(check, want_c, want_q, p, s);
}
}  // namespace abft
