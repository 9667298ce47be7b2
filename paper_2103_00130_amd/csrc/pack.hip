// Encode and pack the weight matrix (Algorithm 1 of arXiv 2103.00130: the rowSum[]
// loop and pack(B, rowSum[]); Section IV-A-3: the checksum is packed together with B
// so that the product kernel sees one encoded matrix).  Runs once per weight.
#include "abft_internal.h"

namespace abft {
namespace {

__device__ inline int8_t load_b(const int8_t* B, int64_t ldb, int transposed, int k, int j, int K, int N) {
    if (k >= K || j >= N) return 0;
    return transposed ? B[(int64_t)j * ldb + k] : B[(int64_t)k * ldb + j];
}

// One thread per 16-byte chunk of the packed layout (16 consecutive k of one column).
__global__ void pack_units_kernel(const int8_t* __restrict__ B, int64_t ldb, int transposed, int K, int N,
                                  int KB, int64_t n_chunks, int8_t* __restrict__ packed) {
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_chunks) return;
    const int c = (int)(q % kUnitN);
    const int kg = (int)((q / kUnitN) % 4);
    const int unit = (int)((q / (kUnitN * 4)) % kUnitsPerTile);
    const int kb = (int)((q / (kUnitN * 4 * kUnitsPerTile)) % KB);
    const int ntile = (int)(q / ((int64_t)kUnitN * 4 * kUnitsPerTile * KB));
    const int j = ntile * kTileN + unit * kUnitN + c;
    const int k0 = kb * kUnitK + kg * 16;
    uint32_t w[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b)
            v |= (uint32_t)(uint8_t)load_b(B, ldb, transposed, k0 + 4 * d + b, j, K, N) << (8 * b);
        w[d] = v;
    }
    reinterpret_cast<uint4*>(packed)[q] = make_uint4(w[0], w[1], w[2], w[3]);
}

// S_B[k] = sum_j B[k][j] (the encoded column, exact int32), one wavefront per k.
// Also emits the four signed base-256 digits of S_B[k]: d0 in [-128,127] with
// s = d0 + 256*s1, and so on; the last digit is s3 reduced to 8 bits, which is exact
// modulo 2^32.  Rows k >= K (padding) get zeros.
__device__ inline void write_digits(int8_t* limbs, int k, int32_t s) {
#pragma unroll
    for (int d = 0; d < kLimbs; ++d) {
        const int32_t dig = (int32_t)(((uint32_t)s + 128u) & 255u) - 128;
        limbs[limb_offset(k, d)] = (int8_t)dig;
        s = (int32_t)((uint32_t)s - (uint32_t)dig) >> 8;
    }
}

// For Algorithm 1 as printed (Section IV-A-2) the same pass also emits rowSum[k] = S_B[k] mod 127
// in [0,126]: as an int32 array and, in the digit layout, as a single live digit column.
__global__ void checksum_rows_kernel(const int8_t* __restrict__ B, int64_t ldb, int transposed, int K, int N,
                                     int Kpad, int32_t* __restrict__ S_B, int8_t* __restrict__ limbs,
                                     int32_t* __restrict__ S_B127, int8_t* __restrict__ limbs127) {
    const int k = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
    const int lane = threadIdx.x % 64;
    if (k >= Kpad) return;
    int32_t s = 0;
    if (k < K)
        for (int j = lane; j < N; j += 64) s += load_b(B, ldb, transposed, k, j, K, N);
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) {
        S_B[k] = s;
        write_digits(limbs, k, s);
        int32_t r = s % 127;
        if (r < 0) r += 127;
        S_B127[k] = r;
        write_digits(limbs127, k, r);
    }
}

// colsum[j] = sum_k B[k][j] (rank-1 term e_k^T B_I of Eq. 1); zeros for padded columns.
// Workgroup (column group of 64, K slice of 256): thread (c, q) sums 64 k-values of column c,
// the four q are combined in LDS and added to colsum (zeroed beforehand) with one integer
// atomic per column and slice; integer addition makes the order irrelevant.
__global__ void colsum_kernel(const int8_t* __restrict__ B, int64_t ldb, int transposed, int K, int N,
                              int32_t* __restrict__ colsum) {
    __shared__ int32_t part[4][64];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + c;
    const int k0 = blockIdx.y * 256 + q * 64;
    int32_t s = 0;
    if (j < N)
        for (int k = k0; k < min(k0 + 64, K); ++k) s += load_b(B, ldb, transposed, k, j, K, N);
    part[q][c] = s;
    __syncthreads();
    if (q == 0 && j < N) {
        s = part[0][c] + part[1][c] + part[2][c] + part[3][c];
        if (s != 0) atomicAdd(&colsum[j], s);
    }
}

// total = sum_k S_B[k] (wrap-around), single workgroup so the result is a plain store.
__global__ void total_kernel(const int32_t* __restrict__ S_B, int Kpad, int32_t* __restrict__ total) {
    __shared__ uint32_t part[256];
    uint32_t s = 0;
    for (int k = threadIdx.x; k < Kpad; k += blockDim.x) s += (uint32_t)S_B[k];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *total = (int32_t)part[0];
}

__global__ void flip_bit_kernel(int8_t* packed, int64_t off, int bit) {
    packed[off] = (int8_t)((uint8_t)packed[off] ^ (uint8_t)(1u << bit));
}

__global__ void flip_checksum_bit_kernel(int32_t* S_B, int8_t* limbs, int32_t* total, int k, int bit) {
    const uint32_t old = (uint32_t)S_B[k];
    const uint32_t now = old ^ (1u << bit);
    S_B[k] = (int32_t)now;
    write_digits(limbs, k, (int32_t)now);
    *total = (int32_t)((uint32_t)*total + (now - old));
}

// the same for the 8-bit column of Algorithm 1 as printed: rowSum[k] is one int8 in memory
__global__ void flip_checksum127_bit_kernel(int32_t* S_B127, int8_t* limbs127, int32_t* total127, int k, int bit) {
    const int32_t old = S_B127[k];
    const int32_t now = (int32_t)(int8_t)((uint8_t)old ^ (uint8_t)(1u << bit));
    S_B127[k] = now;
    write_digits(limbs127, k, now);
    *total127 = (int32_t)((uint32_t)*total127 + ((uint32_t)now - (uint32_t)old));
}

__global__ void fill_zero_kernel(int32_t* p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace

hipError_t launch_pack(const int8_t* B, int64_t ldb, int transposed, abft_packed_b* h, hipStream_t s) {
    const int Kpad = h->KB * kUnitK, Npad = h->NT * kTileN;
    const int64_t n_chunks = (int64_t)h->NT * h->KB * kUnitsPerTile * 4 * kUnitN;
    pack_units_kernel<<<dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, s>>>(
        B, ldb, transposed, h->K, h->N, h->KB, n_chunks, h->packed);
    checksum_rows_kernel<<<dim3((Kpad + 3) / 4), dim3(256), 0, s>>>(B, ldb, transposed, h->K, h->N, Kpad, h->S_B,
                                                                    h->limbs, h->S_B127, h->limbs127);
    fill_zero_kernel<<<dim3((unsigned)((Npad + 255) / 256)), dim3(256), 0, s>>>(h->colsum, (size_t)Npad);
    colsum_kernel<<<dim3((unsigned)(Npad / 64), (unsigned)((h->K + 255) / 256)), dim3(256), 0, s>>>(B, ldb, transposed, h->K, h->N,
                                                                                                  h->colsum);
    total_kernel<<<dim3(1), dim3(256), 0, s>>>(h->S_B, Kpad, h->total);
    total_kernel<<<dim3(1), dim3(256), 0, s>>>(h->S_B127, Kpad, h->total + 1);
    return hipGetLastError();
}

hipError_t launch_flip_bit(abft_packed_b* h, int k, int j, int bit, hipStream_t s) {
    flip_bit_kernel<<<dim3(1), dim3(1), 0, s>>>(h->packed, packed_elem_offset(k, j, h->KB), bit);
    return hipGetLastError();
}

hipError_t launch_flip_checksum_bit(abft_packed_b* h, int k, int bit, hipStream_t s) {
    flip_checksum_bit_kernel<<<dim3(1), dim3(1), 0, s>>>(h->S_B, h->limbs, h->total, k, bit);
    return hipGetLastError();
}

hipError_t launch_flip_checksum127_bit(abft_packed_b* h, int k, int bit, hipStream_t s) {
    flip_checksum127_bit_kernel<<<dim3(1), dim3(1), 0, s>>>(h->S_B127, h->limbs127, h->total + 1, k, bit);
    return hipGetLastError();
}

hipError_t launch_fill_zero(int32_t* p, size_t n_ints, hipStream_t s) {
    if (n_ints == 0) return hipSuccess;
    fill_zero_kernel<<<dim3((unsigned)((n_ints + 255) / 256)), dim3(256), 0, s>>>(p, n_ints);
    return hipGetLastError();
}

}  // namespace abft
