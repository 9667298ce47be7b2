// General-path tiled checked GEMM (any alignment of A): 128x128 tile, 2x2 wavefronts.
#include "gemm_tile_kernel.h"

namespace abft {
hipError_t launch_gemm_tile_g128(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    return tile::launch_cfg<128, 128, 2, 2>(check, want_c, want_q, p, s);
}
}  // namespace abft
