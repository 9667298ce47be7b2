// Internal declarations shared by the HIP translation units of libabftgemm.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace abft {

// ---- packed weight layout -----------------------------------------------------------
// B is cut into "units" of 64 k-values x 32 columns = 2 KiB, stored as
// [k-group kg 0..3][column c 0..31][16 consecutive k bytes].  A 32x32x32 int8 MFMA
// takes k-groups {2h, 2h+1} of a unit as its B operand with lane l reading the
// 16 bytes at h*1024 + l*16; a 16x16x64 MFMA takes columns 16s..16s+15 of all four
// k-groups with lane l reading (l/16)*512 + (16s + l%16)*16.  Units are ordered
// [n-tile of 256 columns][k-block of 64][unit 0..7] so that a workgroup streaming
// along K for one n-tile reads consecutive memory.  Rows k >= K and columns
// j >= N are zero, which leaves both the product and the checksum unchanged.
constexpr int kUnitK = 64;        // k-values per unit
constexpr int kUnitN = 32;        // columns per unit
constexpr int kUnitBytes = kUnitK * kUnitN;
constexpr int kTileN = 256;       // columns per packed n-tile
constexpr int kUnitsPerTile = kTileN / kUnitN;
constexpr int kLimbs = 4;         // signed base-256 digits of an int32 checksum entry

__host__ __device__ inline int64_t packed_unit_offset(int ntile, int kb, int unit, int KB) {
    return (((int64_t)ntile * KB + kb) * kUnitsPerTile + unit) * kUnitBytes;
}
// byte offset of logical B[k][j]
__host__ __device__ inline int64_t packed_elem_offset(int k, int j, int KB) {
    const int ntile = j / kTileN, unit = (j % kTileN) / kUnitN, c = j % kUnitN;
    const int kb = k / kUnitK, kg = (k % kUnitK) / 16, b = k % 16;
    return packed_unit_offset(ntile, kb, unit, KB) + (kg * kUnitN + c) * 16 + b;
}
// Checksum digits: [k-block][k-group][digit 0..3][16 k bytes]; digit d of S_B[k]
// multiplies 256^d.  Same k order as the units, so a 16x16x64 MFMA reads digit
// column d with lane l = kg*16 + d.
__host__ __device__ inline int64_t limb_offset(int k, int digit) {
    const int kb = k / kUnitK, kg = (k % kUnitK) / 16, b = k % 16;
    return (((int64_t)kb * 4 + kg) * kLimbs + digit) * 16 + b;
}

}  // namespace abft

struct abft_packed_b {
    int K, N;
    int KB;            // k-blocks of 64, rounded up to an even count (zero padded)
    int NT;            // n-tiles of 256
    int device;
    int8_t* packed;    // NT*KB*8 units
    int8_t* limbs;     // KB*64*4 bytes
    int32_t* S_B;      // [KB*64], zero past K
    int32_t* colsum;   // [NT*256], zero past N
    int32_t* total;    // [0] sum of S_B (wrap-around), [1] sum of S_B127
    int8_t* limbs127;  // as limbs, for rowSum = S_B mod 127 (digit 0 only)
    int32_t* S_B127;   // [KB*64] S_B mod 127 in [0,126], zero past K
};

namespace abft {

struct RequantDev {
    int32_t zA, zC;
    const float* mult;
    int32_t per_channel;
    const int32_t* bias;
};

#ifdef __HIPCC__
// Requantization of one 32-bit value (Section III-B with the rank-1 correction of Eq. 1 for a
// symmetric B): t = v - zA * colsum (+ bias) in wrap-around int32, one binary32 multiply, round
// to nearest even, + zC, clamp to [0, 255].  The one place this arithmetic is written down.
// What a column contributes, fetched once per column: colsum * zA - bias as one wrap-around term, and the
// multiplier (a kernel that stores between two uses would otherwise have to fetch them again every time).
struct RequantCol {
    uint32_t sub;   // zA * colsum - bias (mod 2^32)
    float mult;
};
__device__ inline RequantCol requant_col(int32_t cs, int col, const RequantDev& rq) {
    RequantCol c;
    c.sub = (uint32_t)rq.zA * (uint32_t)cs;
    if (rq.bias) c.sub -= (uint32_t)rq.bias[col];
    c.mult = rq.mult[rq.per_channel ? col : 0];
    return c;
}
__device__ inline uint8_t requant_with(int32_t v, const RequantCol& c, int32_t zC) {
    const uint32_t t = (uint32_t)v - c.sub;
    const float p = __fmul_rn((float)(int32_t)t, c.mult);
    float y = __builtin_rintf(p) + (float)zC;
    y = fminf(fmaxf(y, 0.0f), 255.0f);
    return (uint8_t)y;
}
__device__ inline uint8_t requant_one(int32_t v, int32_t cs, int col, const RequantDev& rq) {
    return requant_with(v, requant_col(cs, col, rq), rq.zC);
}
#endif

struct GemmParams {
    const uint8_t* A;
    int64_t lda;
    int M, N, K, KB;           // KB: k-blocks of 64 in the packed weight (even)
    int KB2;                   // stages of 128 k-values = KB / 2
    int a_vec_ok;              // A and lda are multiples of 16 bytes
    int mod127;                // compare modulo 127 (Algorithm 1 as printed) instead of 2^32
    int err_accumulate;        // flagged rows are added to *err_count instead of overwriting it
    int share_q, share_r;      // the checksum product's K range (stages or k-blocks) is dealt out to the tile columns /
                               // column blocks of the grid: block c takes share_q units, the first share_r blocks one more
                               // (set by the launcher: a division by a run-time count costs a kernel hundreds of cycles)
    const int8_t* packed;
    const int8_t* limbs;
    const int32_t* colsum;
    const int32_t* total;
    int32_t* C;
    int64_t ldc;
    int32_t* row_flags;
    int32_t* err_count;
    uint8_t* Cq;
    int64_t ldcq;
    RequantDev rq;
    const void* inj;           // abft_inject_t[n_inj]
    int n_inj;
    int ksplit;                // K slices across workgroups (split-K kernels; 1 elsewhere)
    int32_t* ws_tickets;       // split-K: one arrival counter per tile
    int32_t* ws_part;          // split-K: partial tiles, [tile][slice][value][thread]
    size_t ws_ints;            // ints the caller's workspace holds
    unsigned long long* clock_trace;  // diagnostic builds (ABFT_CLOCK_TRACE): 6 words per workgroup, else NULL
    int32_t* ws;               // workspace: counting words in the first kWsHeaderInts ints, then the per-row words
};

constexpr int kWsHeaderInts = 64;   // top arrival word, 16 group arrival words (any-alignment kernel), word of finished rows
constexpr int kTicketGroups = 16;
constexpr int kWsDoneWord = 48;     // int offset, inside the header, of the 64-bit word that counts finished rows (low half)
                                    // and corrupted ones among them (high half): direct-to-LDS tile kernels, streaming kernel
constexpr int kTicketFlatMax = 128;  // grids up to this size count their arrivals on one word
// the streaming kernel spreads its per-row sums over kSmallMSlots slots of kSmallMRows rows
constexpr int kSmallMSlots = 32;
constexpr int kSmallMRows = 64;

// ints of workspace the row words and counting words of a problem with M rows take
inline size_t ws_base_ints(int M) {
    const size_t rows = 2 * ((((size_t)M + 63) / 64) * 64);  // one 64-bit word per row
    // streaming kernel: one 64-bit word per (slot, row) and one per row
    const size_t streaming = 2 * ((size_t)kSmallMSlots * kSmallMRows + kSmallMRows);
    return (size_t)kWsHeaderInts + (rows > streaming ? rows : streaming);
}

// Split-K across workgroups (64x64 tiles, grids that would leave most compute units idle): how many K slices,
// and where the tile tickets and the partial tiles lie in the workspace behind the row words.  One place for
// the rule, so that abft_gemm_workspace_bytes and the launcher agree.
constexpr int kSplitKPartInts = 256 * 17;   // per workgroup: 256 threads x (16 accumulator values + 1 column sum)
struct SplitKPlan {
    int z;                                  // slices (1 = no split)
    size_t tickets_off, part_off, total_ints;
};
inline SplitKPlan splitk_plan(int M, int N, int stages) {
    SplitKPlan pl;
    const long tiles = (long)((M + 63) / 64) * ((N + 63) / 64);
    pl.z = 1;
    // The slices of a tile meet through memory (the L2s are not coherent with each other): store the partial tile,
    // wait for the acknowledgement, take the ticket, fetch the others' partials - three dependent device-scope round
    // trips, measured at 3.5-4 us.  A stage of the unsplit 64x64 loop takes about 0.25 us, so the split pays from
    // about forty stages on (measured: 256x512x4096 8.1 us split against 8.5 unsplit, 256x1024x8192 10.5 against
    // 14.0, 128x128x16384 9.8 against 33.9; 256x512x2048 7.6 against 5.9), and slices of fewer than four stages
    // are all overhead.
    if (stages >= 40)
        for (int z = 16; z >= 2; z >>= 1)
            if (tiles * z <= 256 && stages % z == 0 && stages / z >= 4) {
                pl.z = z;
                break;
            }
    pl.tickets_off = ws_base_ints(M);
    pl.part_off = pl.tickets_off + (size_t)((tiles + 63) / 64 * 64);
    pl.total_ints = pl.z > 1 ? pl.part_off + (size_t)tiles * pl.z * kSplitKPartInts : pl.tickets_off;
    return pl;
}

// first unit of block c's share (see share_q, share_r)
__host__ __device__ inline int share_begin(int c, int q, int r) { return c * q + (c < r ? c : r); }

#ifdef __HIPCC__
// Arrival count of the workgroups of a grid in two levels, so that no workspace word takes more
// than a few dozen atomics at once (hundreds of returned atomics on one address serialise for
// microseconds): a workgroup arrives at the word of its group (block id modulo kTicketGroups) with
// its contribution `mine` in the high half; the last of a group carries the group's sum on to
// the top word (grids of at most kTicketFlatMax workgroups skip the first level).  True for the
// one workgroup that completes the top word, *total then holds the sum over the grid; both levels leave their words at zero.  Everything a workgroup did with
// returned device-scope atomics before it arrives is complete when the last one gets here.
__device__ inline bool arrive_two_level(int32_t* ws, uint32_t mine, uint32_t n_blocks, uint32_t block, uint32_t* total) {
    unsigned long long* const top0 = reinterpret_cast<unsigned long long*>(ws);
    if (n_blocks <= (uint32_t)kTicketFlatMax) {
        // a small grid arrives at the top word directly: one round trip less
        const unsigned long long old0 = __hip_atomic_fetch_add(top0, ((unsigned long long)mine << 32) | 1ull, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)old0 != n_blocks - 1u) return false;
        *total = (uint32_t)(old0 >> 32) + mine;
        __hip_atomic_store(top0, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    const uint32_t g = block & (kTicketGroups - 1);
    const uint32_t n_g = (n_blocks - g + kTicketGroups - 1) / kTicketGroups;
    const uint32_t n_active = n_blocks < (uint32_t)kTicketGroups ? n_blocks : (uint32_t)kTicketGroups;
    unsigned long long* const top = reinterpret_cast<unsigned long long*>(ws);
    unsigned long long* const grp = reinterpret_cast<unsigned long long*>(ws + 16) + g;
    unsigned long long old = __hip_atomic_fetch_add(grp, ((unsigned long long)mine << 32) | 1ull, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
    if ((uint32_t)old != n_g - 1u) return false;
    const uint32_t gsum = (uint32_t)(old >> 32) + mine;
    __hip_atomic_store(grp, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __hip_atomic_fetch_add(top, ((unsigned long long)gsum << 32) | 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((uint32_t)old != n_active - 1u) return false;
    *total = (uint32_t)(old >> 32) + gsum;
    __hip_atomic_store(top, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}
#endif

enum Variant { kTile256 = 1, kTile128 = 2, kTile64 = 3, kSmallM = 4, kTile256w24 = 5, kTile256w42 = 6, kVariantEnd = 7 };

// launchers (each returns the hipError_t of its launch)
hipError_t launch_pack(const int8_t* B, int64_t ldb, int transposed, abft_packed_b* h, hipStream_t s);
hipError_t launch_flip_bit(abft_packed_b* h, int k, int j, int bit, hipStream_t s);
hipError_t launch_flip_checksum_bit(abft_packed_b* h, int k, int bit, hipStream_t s);
hipError_t launch_flip_checksum127_bit(abft_packed_b* h, int k, int bit, hipStream_t s);
hipError_t launch_fill_zero(int32_t* p, size_t n_ints, hipStream_t s);
hipError_t launch_gemm_tile(int variant, bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s);
hipError_t launch_gemm_smallm(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s);
hipError_t launch_requantize(const int32_t* C, int64_t ldc, int M, int N, const int32_t* colsum,
                             const RequantDev& rq, uint8_t* Cq, int64_t ldcq, hipStream_t s);
hipError_t launch_verify_rows(const int32_t* C, int64_t ldc, int M, int N, const int32_t* row_chk,
                              int32_t* row_flags, int32_t* err_count, hipStream_t s);
hipError_t launch_list_flagged(const int32_t* flags, int M, int32_t* idx, int32_t* count, hipStream_t s);
hipError_t launch_gather_rows(const uint8_t* A, int64_t lda, const int32_t* idx, int n, int K, uint8_t* A2,
                              int64_t lda2, hipStream_t s);
hipError_t launch_scatter_rows(const int32_t* C2, const uint8_t* Cq2, const int32_t* flags2, const int32_t* idx, int n,
                               int N, int32_t* C, int64_t ldc, uint8_t* Cq, int64_t ldcq, int32_t* flags, hipStream_t s);
hipError_t launch_add_int(int32_t* dst, const int32_t* src, hipStream_t s);
hipError_t launch_gather_rows_bounded(const uint8_t* A, int64_t lda, const int32_t* idx, const int32_t* count, int limit, int K,
                                      uint8_t* A2, int64_t lda2, hipStream_t s);
hipError_t launch_scatter_rows_bounded(const int32_t* C2, const uint8_t* Cq2, const int32_t* flags2, const int32_t* idx,
                                       const int32_t* count, int limit, int N, int32_t* C, int64_t ldc, uint8_t* Cq, int64_t ldcq,
                                       int32_t* flags, hipStream_t s);
hipError_t launch_recount(const int32_t* count, const int32_t* cnt2, int limit, int32_t* err_count, int32_t* status,
                          hipStream_t s);
hipError_t launch_locate_correct(const uint8_t* A, int64_t lda, int M, const abft_packed_b* h, int32_t* C, int64_t ldc,
                                 int32_t* row_flags, int32_t* err_count, const RequantDev* rq, uint8_t* Cq, int64_t ldcq,
                                 int32_t* col_flags, int32_t* report, int32_t* scratch, hipStream_t s);
hipError_t launch_calib_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
hipError_t launch_clock_probe(unsigned long long* out, unsigned long long ticks, hipStream_t s);
hipError_t launch_mfma_peak_probe(unsigned long long* out, int iters, hipStream_t s);
hipError_t launch_row_checksum(const uint8_t* A, int64_t lda, int M, int K, const int32_t* S_B,
                               int32_t* row_chk, hipStream_t s);

// EmbeddingBag: lookups from which the batch kernel is chosen over the group kernel, by the number of
// 16-byte pieces of a row's codes
constexpr int64_t eb_batch_min_lookups(int pieces) {
    return pieces <= 1 ? 49152 : pieces == 2 ? 32768 : pieces == 4 ? 98304 : pieces == 8 ? 262144 : pieces == 16 ? 7168 : 16384;
}

// Lets `kern` use `bytes` of dynamic LDS on the current device: the attribute belongs to the device, so it
// is set once per device and kernel (`done`: one bit per device ordinal, shared by the threads of the host)
inline hipError_t allow_dynamic_lds(const void* kern, size_t bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// records `code` and a message for abft_last_error(); returns `code`
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace abft
