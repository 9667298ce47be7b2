// Dispatch of the tiled checked GEMM over its compiled tile shapes.
#include "abft_internal.h"

namespace abft {
#define ABFT_DECL(name) hipError_t launch_gemm_tile_##name(bool, bool, bool, const GemmParams&, hipStream_t)
ABFT_DECL(a256);
ABFT_DECL(a256w24);
ABFT_DECL(a256w42);
ABFT_DECL(a128);
ABFT_DECL(a64);
ABFT_DECL(a64r8);
ABFT_DECL(a64r4);
ABFT_DECL(a64s);
ABFT_DECL(a64k2);
ABFT_DECL(g128);
ABFT_DECL(g64);
#undef ABFT_DECL

hipError_t launch_gemm_tile(int variant, bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    // direct-to-LDS kernels need whole, aligned 16-byte chunks of A
    // (and 32-bit byte offsets into A)
    const bool fast_a = p.a_vec_ok && (p.K % 16 == 0) && ((int64_t)(p.M - 1) * p.lda + p.K <= 0x7fffffffll);
    if (!fast_a) {
        if (p.mod127) return hipErrorNotSupported;
        if (variant == kTile64) return launch_gemm_tile_g64(check, want_c, want_q, p, s);
        return launch_gemm_tile_g128(check, want_c, want_q, p, s);
    }
    switch (variant) {
        case kTile256: return launch_gemm_tile_a256(check, want_c, want_q, p, s);
        case kTile128: return launch_gemm_tile_a128(check, want_c, want_q, p, s);
        case kTile64: {
            // The 64x64 kernels are bound by instruction issue and the LDS reads of a wavefront, not by
            // the matrix cores, so they run as four wavefronts of 32x32 on four SIMDs (5-10 % faster than
            // two of 32x64).  At most one workgroup per compute unit and a long K loop: K is split between
            // two such groups of wavefronts, so that every SIMD has two wavefronts to issue from (10-15 %
            // faster from K = 1536 on: 1024x1024x4096 unchecked 11.7 -> 10.4 us, 512x1024x4096 10.9 -> 8.9;
            // slower at K <= 1024, where the hand-over at the end costs more than the loop gains; four
            // groups, or four lone wavefronts of 64x64, are slower than two groups).  The launcher refuses
            // a K that does not split evenly or whose checksum share per tile column is too long for the
            // staged digits; then one group with a ring of eight stages takes a long K (it takes most of
            // a unit's LDS, and filling it costs more than it saves below about sixteen stages).
            const int64_t tiles = (int64_t)((p.M + 63) / 64) * ((p.N + 63) / 64);
            // few tiles and a long K: K is split across workgroups as well, so that the compute units that would sit
            // idle take slices of it (the launcher refuses when the caller's workspace has no room for the partial tiles)
            if (splitk_plan(p.M, p.N, p.KB2).z > 1) {
                const hipError_t e = launch_gemm_tile_a64s(check, want_c, want_q, p, s);
                if (e != hipErrorNotSupported) return e;
            }
            if (tiles <= 256 && p.K >= 1536) {
                const hipError_t e = launch_gemm_tile_a64k2(check, want_c, want_q, p, s);
                if (e != hipErrorNotSupported) return e;
            }
            if (tiles <= 256 && p.K >= 2048) return launch_gemm_tile_a64r8(check, want_c, want_q, p, s);
            // short K on such a grid: a ring of four stages, all in flight before the first k-step, instead of the
            // double buffer whose every stage waits out a trip to memory (a few tenths of a microsecond at 256x512x1024)
            if (tiles <= 256 && p.K > 256) return launch_gemm_tile_a64r4(check, want_c, want_q, p, s);
            return launch_gemm_tile_a64(check, want_c, want_q, p, s);
        }
        case kTile256w24: return launch_gemm_tile_a256w24(check, want_c, want_q, p, s);
        case kTile256w42: return launch_gemm_tile_a256w42(check, want_c, want_q, p, s);
        default: return hipErrorInvalidValue;
    }
}
}  // namespace abft
