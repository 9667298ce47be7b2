// Direct-to-LDS tiled checked GEMM: 64x64 workgroup tile, 2x1 wavefronts, a ring of eight stages.
// For grids that leave at most one workgroup per compute unit: the K loop of such a launch is bound
// by the latency of its loads, and eight stages in flight instead of two hide most of it.
#include "gemm_tile_async.h"

namespace abft {
hipError_t launch_gemm_tile_a64s8(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    return atile::launch_cfg<64, 64, 2, 1, 8>(check, want_c, want_q, p, s);
}
}  // namespace abft
