// Bandwidth-bound companions of the checked GEMM: stand-alone requantization
// (Section III-B of arXiv 2103.00130), re-verification of a stored C_temp against the
// checksum column (Eq. 2b; the paper's "bit flip in the 32-bit intermediate" fault
// model applied to a matrix at rest), and the checksum column A*S_B on its own.
#include "abft_internal.h"

#include <algorithm>

namespace abft {
namespace {

// 4 consecutive columns per thread: one 16-byte load of C, one 4-byte store of Cq when
// the row is aligned for it, element-wise otherwise.
__global__ void requantize_kernel(const int32_t* __restrict__ C, int64_t ldc, int M, int N,
                                  const int32_t* __restrict__ colsum, RequantDev rq, uint8_t* __restrict__ Cq,
                                  int64_t ldcq) {
    const int j0 = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (j0 >= N) return;
    const int n = min(4, N - j0);
    // rows in strides of the grid's second dimension (which the hardware caps at 65535)
    for (int row = blockIdx.y; row < M; row += gridDim.y)
        for (int e = 0; e < n; ++e) {
            const int col = j0 + e;
            Cq[(int64_t)row * ldcq + col] = requant_one(C[(int64_t)row * ldc + col], colsum[col], col, rq);
        }
}

// one workgroup (256 lanes) per row: tSum, comparison with row_chk, flag, count.
__global__ void verify_rows_kernel(const int32_t* __restrict__ C, int64_t ldc, int M, int N,
                                   const int32_t* __restrict__ row_chk, int32_t* __restrict__ row_flags,
                                   int32_t* __restrict__ err_count) {
    __shared__ uint32_t part[4];
    const int row = blockIdx.x;
    uint32_t s = 0;
    for (int j = threadIdx.x; j < N; j += blockDim.x) s += (uint32_t)C[(int64_t)row * ldc + j];
    for (int off = 32; off > 0; off >>= 1) s += (uint32_t)__shfl_xor((int)s, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t t = part[0] + part[1] + part[2] + part[3];
        const int f = ((int32_t)t != row_chk[row]) ? 1 : 0;
        row_flags[row] = f;
        if (err_count && f) atomicAdd(err_count, 1);
    }
}

// chk[i] = sum_k A[i][k] * S_B[k], wrap-around int32; one wavefront per row.
__global__ void row_checksum_kernel(const uint8_t* __restrict__ A, int64_t lda, int M, int K,
                                    const int32_t* __restrict__ S_B, int32_t* __restrict__ row_chk) {
    const int row = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
    const int lane = threadIdx.x & 63;
    if (row >= M) return;
    uint32_t s = 0;
    for (int k = lane; k < K; k += 64) s += (uint32_t)A[(int64_t)row * lda + k] * (uint32_t)S_B[k];
    for (int off = 32; off > 0; off >>= 1) s += (uint32_t)__shfl_xor((int)s, off);
    if (lane == 0) row_chk[row] = (int32_t)s;
}

// Plain grid-stride copy of 16-byte words: the known-size reference against which the
// memory-traffic counters of a profiler are scaled.
__global__ void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// One lane reads the shader-clock cycle counter and the constant-rate (100 MHz) wall counter, idles until the
// wall counter has advanced by `ticks`, and reads both again: cycles over wall time is the shader clock the
// chip ran at in between.  Launched on a second stream it measures the clock under whatever else is running.
// The wall counter advances on its own, so the wait always ends.
__global__ void clock_probe_kernel(unsigned long long* __restrict__ out, unsigned long long ticks) {
    if (threadIdx.x != 0) return;
    const unsigned long long r0 = wall_clock64(), c0 = clock64();
    while (wall_clock64() - r0 < ticks) __builtin_amdgcn_s_sleep(16);
    const unsigned long long r1 = wall_clock64(), c1 = clock64();
    out[0] = r0;
    out[1] = c0;
    out[2] = r1;
    out[3] = c1;
}

// Register-only matrix-core load: every wavefront runs `iters` rounds of four independent 32x32x32 int8 MFMAs on
// operands that never leave its registers (no LDS, no memory).  The first thread of every workgroup records the
// shader-clock cycle counter and the 100 MHz wall counter around the loop: what the matrix cores deliver, and
// at which clock, when nothing but they draws power.  Four wavefronts per workgroup, one per SIMD.
typedef int probe_v4i __attribute__((ext_vector_type(4)));
typedef int probe_v16i __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void mfma_peak_probe_kernel(unsigned long long* __restrict__ out, int iters) {
    probe_v16i acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0;
    const int t = (int)threadIdx.x;
    const probe_v4i a = {t, t + 1, t + 2, t + 3}, b = {t * 3, t * 5, t * 7, t * 9};
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
    }
    int keep = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) keep ^= acc[i][e];
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    if (threadIdx.x == 0 || keep == 0x7fffffff) {   // (the second condition only keeps the result alive)
        unsigned long long* const o = out + (size_t)blockIdx.x * 4;
        o[0] = c0;
        o[1] = r0;
        o[2] = c1;
        o[3] = r1;
    }
}

// Recovery helpers: list the flagged rows, gather them, put recomputed rows back.
__global__ void list_flagged_kernel(const int32_t* __restrict__ flags, int M, int32_t* __restrict__ idx,
                                    int32_t* __restrict__ count) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < M && flags[r] != 0) idx[atomicAdd(count, 1)] = r;   // any order will do
}

__global__ void gather_rows_kernel(const uint8_t* __restrict__ A, int64_t lda, const int32_t* __restrict__ idx,
                                   int K, uint8_t* __restrict__ A2, int64_t lda2) {
    const uint8_t* src = A + (int64_t)idx[blockIdx.x] * lda;
    uint8_t* dst = A2 + (int64_t)blockIdx.x * lda2;
    for (int k = threadIdx.x; k < (int)lda2; k += blockDim.x) dst[k] = k < K ? src[k] : (uint8_t)0;
}

__global__ void scatter_rows_kernel(const int32_t* __restrict__ C2, const uint8_t* __restrict__ Cq2,
                                    const int32_t* __restrict__ flags2, const int32_t* __restrict__ idx, int N,
                                    int32_t* __restrict__ C, int64_t ldc, uint8_t* __restrict__ Cq, int64_t ldcq,
                                    int32_t* __restrict__ flags) {
    const int r = idx[blockIdx.x];
    for (int j = threadIdx.x; j < N; j += blockDim.x) {
        if (C) C[(int64_t)r * ldc + j] = C2[(int64_t)blockIdx.x * N + j];
        if (Cq) Cq[(int64_t)r * ldcq + j] = Cq2[(int64_t)blockIdx.x * N + j];
    }
    if (threadIdx.x == 0) flags[r] = flags2[blockIdx.x];
}

__global__ void add_int_kernel(int32_t* dst, const int32_t* src) { *dst += *src; }

// The same helpers with the number of listed rows read on the device (nothing goes back to the host):
// block b of a grid of `limit` blocks handles listed row b if there is one, and otherwise clears its row of
// the gathered operand (so that the product over all `limit` rows is defined and its spare rows pass).
__global__ void gather_rows_bounded_kernel(const uint8_t* __restrict__ A, int64_t lda, const int32_t* __restrict__ idx,
                                           const int32_t* __restrict__ count, int K, uint8_t* __restrict__ A2, int64_t lda2) {
    const bool live = (int)blockIdx.x < *count;
    const uint8_t* src = A + (int64_t)(live ? idx[blockIdx.x] : 0) * lda;
    uint8_t* dst = A2 + (int64_t)blockIdx.x * lda2;
    for (int k = threadIdx.x; k < (int)lda2; k += blockDim.x) dst[k] = (live && k < K) ? src[k] : (uint8_t)0;
}

__global__ void scatter_rows_bounded_kernel(const int32_t* __restrict__ C2, const uint8_t* __restrict__ Cq2,
                                            const int32_t* __restrict__ flags2, const int32_t* __restrict__ idx,
                                            const int32_t* __restrict__ count, int N, int32_t* __restrict__ C, int64_t ldc,
                                            uint8_t* __restrict__ Cq, int64_t ldcq, int32_t* __restrict__ flags) {
    if ((int)blockIdx.x >= *count) return;
    const int r = idx[blockIdx.x];
    for (int j = threadIdx.x; j < N; j += blockDim.x) {
        if (C) C[(int64_t)r * ldc + j] = C2[(int64_t)blockIdx.x * N + j];
        if (Cq) Cq[(int64_t)r * ldcq + j] = Cq2[(int64_t)blockIdx.x * N + j];
    }
    if (threadIdx.x == 0) flags[r] = flags2[blockIdx.x];
}

// status[0] = rows found flagged, status[1] = rows still flagged: those recomputed and flagged again
// (cnt2 counts them: spare rows are all-zero and pass) plus those beyond the limit, which were not touched
__global__ void recount_kernel(const int32_t* __restrict__ count, const int32_t* __restrict__ cnt2, int limit,
                               int32_t* __restrict__ err_count, int32_t* __restrict__ status) {
    const int found = *count, left = (found > limit ? found - limit : 0) + *cnt2;
    if (err_count) *err_count = left;
    if (status) {
        status[0] = found;
        status[1] = left;
    }
}

}  // namespace

hipError_t launch_list_flagged(const int32_t* flags, int M, int32_t* idx, int32_t* count, hipStream_t s) {
    hipError_t e = launch_fill_zero(count, 1, s);
    if (e != hipSuccess) return e;
    list_flagged_kernel<<<dim3((unsigned)((M + 255) / 256)), dim3(256), 0, s>>>(flags, M, idx, count);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const uint8_t* A, int64_t lda, const int32_t* idx, int n, int K, uint8_t* A2,
                              int64_t lda2, hipStream_t s) {
    gather_rows_kernel<<<dim3((unsigned)n), dim3(256), 0, s>>>(A, lda, idx, K, A2, lda2);
    return hipGetLastError();
}

hipError_t launch_scatter_rows(const int32_t* C2, const uint8_t* Cq2, const int32_t* flags2, const int32_t* idx, int n,
                               int N, int32_t* C, int64_t ldc, uint8_t* Cq, int64_t ldcq, int32_t* flags, hipStream_t s) {
    scatter_rows_kernel<<<dim3((unsigned)n), dim3(256), 0, s>>>(C2, Cq2, flags2, idx, N, C, ldc, Cq, ldcq, flags);
    return hipGetLastError();
}

hipError_t launch_add_int(int32_t* dst, const int32_t* src, hipStream_t s) {
    add_int_kernel<<<dim3(1), dim3(1), 0, s>>>(dst, src);
    return hipGetLastError();
}

hipError_t launch_gather_rows_bounded(const uint8_t* A, int64_t lda, const int32_t* idx, const int32_t* count, int limit, int K,
                                      uint8_t* A2, int64_t lda2, hipStream_t s) {
    gather_rows_bounded_kernel<<<dim3((unsigned)limit), dim3(256), 0, s>>>(A, lda, idx, count, K, A2, lda2);
    return hipGetLastError();
}

hipError_t launch_scatter_rows_bounded(const int32_t* C2, const uint8_t* Cq2, const int32_t* flags2, const int32_t* idx,
                                       const int32_t* count, int limit, int N, int32_t* C, int64_t ldc, uint8_t* Cq, int64_t ldcq,
                                       int32_t* flags, hipStream_t s) {
    scatter_rows_bounded_kernel<<<dim3((unsigned)limit), dim3(256), 0, s>>>(C2, Cq2, flags2, idx, count, N, C, ldc, Cq, ldcq, flags);
    return hipGetLastError();
}

hipError_t launch_recount(const int32_t* count, const int32_t* cnt2, int limit, int32_t* err_count, int32_t* status,
                          hipStream_t s) {
    recount_kernel<<<dim3(1), dim3(1), 0, s>>>(count, cnt2, limit, err_count, status);
    return hipGetLastError();
}

hipError_t launch_calib_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 16);
    calib_copy_kernel<<<dim3(grid), dim3(256), 0, s>>>((const uint4*)src, (uint4*)dst, n16);
    return hipGetLastError();
}

hipError_t launch_clock_probe(unsigned long long* out, unsigned long long ticks, hipStream_t s) {
    clock_probe_kernel<<<dim3(1), dim3(64), 0, s>>>(out, ticks);
    return hipGetLastError();
}

hipError_t launch_mfma_peak_probe(unsigned long long* out, int iters, hipStream_t s) {
    mfma_peak_probe_kernel<<<dim3(256), dim3(256), 0, s>>>(out, iters);
    return hipGetLastError();
}

hipError_t launch_requantize(const int32_t* C, int64_t ldc, int M, int N, const int32_t* colsum,
                             const RequantDev& rq, uint8_t* Cq, int64_t ldcq, hipStream_t s) {
    const dim3 block(64), grid((unsigned)((N + 255) / 256), (unsigned)std::min(M, 65535));
    requantize_kernel<<<grid, block, 0, s>>>(C, ldc, M, N, colsum, rq, Cq, ldcq);
    return hipGetLastError();
}

hipError_t launch_verify_rows(const int32_t* C, int64_t ldc, int M, int N, const int32_t* row_chk,
                              int32_t* row_flags, int32_t* err_count, hipStream_t s) {
    if (err_count) {
        hipError_t e = launch_fill_zero(err_count, 1, s);
        if (e != hipSuccess) return e;
    }
    verify_rows_kernel<<<dim3((unsigned)M), dim3(256), 0, s>>>(C, ldc, M, N, row_chk, row_flags, err_count);
    return hipGetLastError();
}

hipError_t launch_row_checksum(const uint8_t* A, int64_t lda, int M, int K, const int32_t* S_B,
                               int32_t* row_chk, hipStream_t s) {
    row_checksum_kernel<<<dim3((unsigned)((M + 3) / 4)), dim3(256), 0, s>>>(A, lda, M, K, S_B, row_chk);
    return hipGetLastError();
}

}  // namespace abft
