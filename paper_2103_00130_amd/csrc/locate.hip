// Locating and correcting a single faulty element of C_temp: the column check of Eq. 2a and the two
// correction formulas of Section IV of arXiv 2103.00130, as an on-demand companion of the checked GEMM.
//
// The method keeps the product itself to detection with an encoded B only (Section IV-A-1: encoding A
// as well is what the paper leaves out for its cost).  Here the other half of the classic scheme runs
// only once a launch has flagged a row: S_A = e^T A is formed from the A in memory, the checksum row
// C'[m][:] = S_A B from the packed B, the column sums of the stored C_temp are compared with it
// (Eq. 2a), and when exactly one row (Eq. 2b, the verdicts the GEMM returned) and exactly one column
// are violated, the element where they cross is recomputed from the column formula, cross-checked with
// the row formula, and written back.  All sums are wrap-around int32, like the row check.
//
// Four small bandwidth-bound kernels (one pass over A, one over the packed B, one over C) and a
// single-workgroup decision kernel; nothing synchronises, nothing is allocated.
#include "../../include/abft_gemm.h"
#include "abft_internal.h"

namespace abft {
namespace {

// S_A[k] += sum of A[i][k] over this block's rows.  A block owns 256 columns and kColsumRows rows: thread
// (kc, rl) walks the rows rl, rl + 16, ... of the block with the 16 columns of chunk kc (one 16-byte load when
// the caller's A allows it - base and lda multiples of 16 - byte by byte otherwise), the sixteen row lanes
// meet in LDS, and one atomic per column and block adds the block's sum.
constexpr int kColsumRows = 256;
__global__ __launch_bounds__(256) void a_colsum_kernel(const uint8_t* __restrict__ A, int64_t lda, int M, int K, int vec_ok,
                                                       int32_t* __restrict__ S_A) {
    __shared__ uint32_t part[16][257];
    const int kc = threadIdx.x & 15, rl = threadIdx.x >> 4;
    const int k0 = blockIdx.x * 256 + kc * 16;
    uint32_t s[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) s[b] = 0;
    // (row blocks in strides of the grid's second dimension, which the hardware caps at 65535)
    for (int64_t r0 = (int64_t)blockIdx.y * kColsumRows; r0 < M; r0 += (int64_t)gridDim.y * kColsumRows) {
        const int r1 = (int)min(r0 + kColsumRows, (int64_t)M);
        if (vec_ok && k0 + 16 <= K) {
            for (int r = (int)r0 + rl; r < r1; r += 16) {
                const uint4 v = *reinterpret_cast<const uint4*>(A + (int64_t)r * lda + k0);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int b = 0; b < 16; ++b) s[b] += (w[b >> 2] >> (8 * (b & 3))) & 0xFFu;
            }
        } else {
            for (int r = (int)r0 + rl; r < r1; r += 16)
#pragma unroll
                for (int b = 0; b < 16; ++b)
                    if (k0 + b < K) s[b] += A[(int64_t)r * lda + k0 + b];
        }
    }
#pragma unroll
    for (int b = 0; b < 16; ++b) part[rl][kc * 16 + b] = s[b];
    __syncthreads();
    const int k = blockIdx.x * 256 + threadIdx.x;
    uint32_t t = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) t += part[q][threadIdx.x];
    if (k < K && t != 0) atomicAdd(&S_A[k], (int32_t)t);
}

// col_chk[j] += sum over this block's k-blocks of S_A[k] * B[k][j], straight from the packed weight.
// A block owns one unit column (32 columns of one n-tile) and the k-blocks kb = by, by + gridDim.y, ...;
// thread (c, kg, h) reads the 16 k-values of column c, k-group kg of every second of those k-blocks
// (one 16-byte load: 32 lanes cover 512 contiguous bytes) against the matching 16 entries of S_A.
__global__ __launch_bounds__(256) void col_checksum_kernel(const int8_t* __restrict__ packed, int KB,
                                                           const int32_t* __restrict__ S_A, int32_t* __restrict__ col_chk) {
    __shared__ uint32_t part[8][32];
    const int c = threadIdx.x & 31, kg = (threadIdx.x >> 5) & 3, h = threadIdx.x >> 7;
    const int ntile = blockIdx.x / kUnitsPerTile, unit = blockIdx.x % kUnitsPerTile;
    uint32_t s = 0;
    for (int kb = blockIdx.y * 2 + h; kb < KB; kb += gridDim.y * 2) {
        const int4 v = *reinterpret_cast<const int4*>(packed + packed_unit_offset(ntile, kb, unit, KB) + (kg * kUnitN + c) * 16);
        const int32_t w[4] = {v.x, v.y, v.z, v.w};
        const int4* sa4 = reinterpret_cast<const int4*>(S_A + kb * kUnitK + kg * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int4 a = sa4[q];
            const int32_t sa[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
            for (int b = 0; b < 4; ++b) s += (uint32_t)sa[b] * (uint32_t)(int32_t)(int8_t)(w[q] >> (8 * b));
        }
    }
    part[threadIdx.x >> 5][c] = s;
    __syncthreads();
    if (threadIdx.x < 32) {
        uint32_t t = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) t += part[q][c];
        if (t != 0) atomicAdd(&col_chk[ntile * kTileN + unit * kUnitN + c], (int32_t)t);
    }
}

// csum[j] += sum of C[i][j] over this block's rows; one column per thread, rows read coalesced.
constexpr int kColsumCRows = 32;
__global__ __launch_bounds__(256) void c_colsum_kernel(const int32_t* __restrict__ C, int64_t ldc, int M, int N,
                                                       int32_t* __restrict__ csum) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= N) return;
    uint32_t s = 0;
    for (int64_t r0 = (int64_t)blockIdx.y * kColsumCRows; r0 < M; r0 += (int64_t)gridDim.y * kColsumCRows) {
        const int r1 = (int)min(r0 + kColsumCRows, (int64_t)M);
        for (int r = (int)r0; r < r1; ++r) s += (uint32_t)C[(int64_t)r * ldc + j];
    }
    if (s != 0) atomicAdd(&csum[j], (int32_t)s);
}

// block-wide sum of one uint32 per thread (1024 threads); every thread gets the total
__device__ inline uint32_t block_sum(uint32_t v, uint32_t* sh) {
    for (int off = 32; off > 0; off >>= 1) v += (uint32_t)__shfl_xor((int)v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t t = 0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += sh[w];
    return t;
}

// The decision and the repair, one workgroup.  report: abft_locate_t.
__global__ __launch_bounds__(1024) void locate_decide_kernel(const uint8_t* __restrict__ A, int64_t lda, int M, int N, int K,
                                                             const int32_t* __restrict__ S_B, const int32_t* __restrict__ col_chk,
                                                             const int32_t* __restrict__ csum, int32_t* __restrict__ C, int64_t ldc,
                                                             int32_t* __restrict__ row_flags, int32_t* __restrict__ err_count,
                                                             int want_q, RequantDev rq, const int32_t* __restrict__ colsum_b,
                                                             uint8_t* __restrict__ Cq, int64_t ldcq, int32_t* __restrict__ col_flags,
                                                             int32_t* __restrict__ report) {
    __shared__ uint32_t sh[16];
    __shared__ int s_row, s_col;
    if (threadIdx.x == 0) s_row = s_col = -1;
    __syncthreads();
    uint32_t n_rows = 0, n_cols = 0;
    for (int i = threadIdx.x; i < M; i += blockDim.x)
        if (row_flags[i] != 0) {
            ++n_rows;
            atomicMax(&s_row, i);
        }
    for (int j = threadIdx.x; j < N; j += blockDim.x) {
        const int f = csum[j] != col_chk[j];
        if (col_flags) col_flags[j] = f;
        if (f) {
            ++n_cols;
            atomicMax(&s_col, j);
        }
    }
    n_rows = block_sum(n_rows, sh);
    n_cols = block_sum(n_cols, sh);
    const int row = s_row, col = s_col;
    int status = (n_rows == 0 && n_cols == 0) ? ABFT_LOCATE_CLEAN : ABFT_LOCATE_NOT_ONE_ELEMENT;
    int32_t old_v = 0, new_v = 0;
    if (n_rows == 1 && n_cols == 1) {
        // first formula: the checksum row's entry minus the other elements of the column;
        // second formula: the checksum column's entry (A S_B)[row] minus the other elements of the row
        uint32_t chk = 0, others = 0;
        for (int k = threadIdx.x; k < K; k += blockDim.x) chk += (uint32_t)A[(int64_t)row * lda + k] * (uint32_t)S_B[k];
        for (int p = threadIdx.x; p < N; p += blockDim.x)
            if (p != col) others += (uint32_t)C[(int64_t)row * ldc + p];
        chk = block_sum(chk, sh);
        others = block_sum(others, sh);
        old_v = C[(int64_t)row * ldc + col];
        const int32_t by_column = (int32_t)((uint32_t)col_chk[col] - ((uint32_t)csum[col] - (uint32_t)old_v));
        const int32_t by_row = (int32_t)(chk - others);
        if (by_column == by_row) {
            status = ABFT_LOCATE_CORRECTED;
            new_v = by_column;
            __syncthreads();  // every thread has read what it needs of the row
            if (threadIdx.x == 0) {
                C[(int64_t)row * ldc + col] = new_v;
                if (want_q) Cq[(int64_t)row * ldcq + col] = requant_one(new_v, colsum_b[col], col, rq);
                row_flags[row] = 0;
                if (err_count) *err_count -= 1;
            }
        }
    }
    if (threadIdx.x == 0) {
        report[0] = status;
        report[1] = status == ABFT_LOCATE_CORRECTED ? row : -1;
        report[2] = status == ABFT_LOCATE_CORRECTED ? col : -1;
        report[3] = status == ABFT_LOCATE_CORRECTED ? old_v : 0;
        report[4] = new_v;
        report[5] = (int32_t)n_rows;
        report[6] = (int32_t)n_cols;
        report[7] = 0;
    }
}

}  // namespace

hipError_t launch_locate_correct(const uint8_t* A, int64_t lda, int M, const abft_packed_b* h, int32_t* C, int64_t ldc,
                                 int32_t* row_flags, int32_t* err_count, const RequantDev* rq, uint8_t* Cq, int64_t ldcq,
                                 int32_t* col_flags, int32_t* report, int32_t* scratch, hipStream_t s) {
    const int K = h->K, N = h->N, Kpad = h->KB * kUnitK, Npad = h->NT * kTileN;
    int32_t* const S_A = scratch;              // [Kpad], zero past K
    int32_t* const col_chk = S_A + Kpad;       // [Npad]
    int32_t* const csum = col_chk + Npad;      // [Npad]
    hipError_t e = launch_fill_zero(scratch, (size_t)Kpad + 2 * (size_t)Npad, s);
    if (e != hipSuccess) return e;
    const int vec_ok = (((uintptr_t)A | (uintptr_t)lda) & 15) == 0;
    a_colsum_kernel<<<dim3((unsigned)((K + 255) / 256), (unsigned)min((M + kColsumRows - 1) / kColsumRows, 65535)), dim3(256), 0, s>>>(
        A, lda, M, K, vec_ok, S_A);
    c_colsum_kernel<<<dim3((unsigned)((N + 255) / 256), (unsigned)min((M + kColsumCRows - 1) / kColsumCRows, 65535)), dim3(256), 0, s>>>(
        C, ldc, M, N, csum);
    // enough blocks along K to fill the chip, at least four k-blocks each
    const int units = h->NT * kUnitsPerTile;
    int ky = (1024 + units - 1) / units;
    ky = ky < 1 ? 1 : ky;
    while (ky > 1 && h->KB / (2 * ky) < 2) --ky;
    col_checksum_kernel<<<dim3((unsigned)units, (unsigned)ky), dim3(256), 0, s>>>(h->packed, h->KB, S_A, col_chk);
    RequantDev none{};
    locate_decide_kernel<<<dim3(1), dim3(1024), 0, s>>>(A, lda, M, N, K, h->S_B, col_chk, csum, C, ldc, row_flags, err_count,
                                                        rq != nullptr, rq ? *rq : none, h->colsum, Cq, ldcq, col_flags, report);
    return hipGetLastError();
}

}  // namespace abft
