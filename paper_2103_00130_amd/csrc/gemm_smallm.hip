// Streaming checked GEMM for M <= 64 (placeholder until the kernel lands).
#include "abft_internal.h"

namespace abft {
hipError_t launch_gemm_smallm(bool, bool, bool, const GemmParams&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace abft
