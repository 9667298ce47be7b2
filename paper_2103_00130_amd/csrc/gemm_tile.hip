// Dispatch of the tiled checked GEMM over its compiled tile shapes.
#include "abft_internal.h"

namespace abft {
hipError_t launch_gemm_tile_t256(bool, bool, bool, const GemmParams&, hipStream_t);
hipError_t launch_gemm_tile_t256w24(bool, bool, bool, const GemmParams&, hipStream_t);
hipError_t launch_gemm_tile_t256w42(bool, bool, bool, const GemmParams&, hipStream_t);
hipError_t launch_gemm_tile_t128(bool, bool, bool, const GemmParams&, hipStream_t);
hipError_t launch_gemm_tile_t64(bool, bool, bool, const GemmParams&, hipStream_t);

hipError_t launch_gemm_tile(int variant, bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    switch (variant) {
        case kTile256: return launch_gemm_tile_t256(check, want_c, want_q, p, s);
        case kTile128: return launch_gemm_tile_t128(check, want_c, want_q, p, s);
        case kTile64: return launch_gemm_tile_t64(check, want_c, want_q, p, s);
        case kTile256w24: return launch_gemm_tile_t256w24(check, want_c, want_q, p, s);
        case kTile256w42: return launch_gemm_tile_t256w42(check, want_c, want_q, p, s);
        default: return hipErrorInvalidValue;
    }
}
}  // namespace abft
