// Direct-to-LDS tiled checked GEMM: 64x64 workgroup tile, 2x2 wavefronts, a ring of four stages, K split across
// workgroups (grids of few tiles and a long K: the slices of a tile meet through the workspace).
#include "gemm_tile_async.h"

namespace abft {
hipError_t launch_gemm_tile_a64s(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    return atile::launch_cfg<64, 64, 2, 2, 4, 1, true>(check, want_c, want_q, p, s);
}
}  // namespace abft
