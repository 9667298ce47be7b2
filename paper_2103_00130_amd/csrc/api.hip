// C ABI of libabftgemm (see include/abft_gemm.h): argument checks, variant choice and
// kernel launches.  No arithmetic of the method happens on the host.
#include <cstdarg>
#include <cstdio>
#include <atomic>
#include <cstring>
#include <new>

#include "../../include/abft_gemm.h"
#include "abft_internal.h"

namespace {

thread_local char g_err[512] = "";
#ifdef ABFT_CLOCK_TRACE
std::atomic<unsigned long long*> g_clock_trace{nullptr};  // set by abft_clock_trace, handed to every tiled launch
#endif

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(ABFT_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(expr)                                      \
    do {                                                   \
        hipError_t e_ = (expr);                            \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);  \
    } while (0)

void free_handle(abft_packed_b* h) {
    if (!h) return;
    (void)hipFree(h->packed);
    (void)hipFree(h->limbs);
    (void)hipFree(h->S_B);
    (void)hipFree(h->colsum);
    (void)hipFree(h->total);
    (void)hipFree(h->limbs127);
    (void)hipFree(h->S_B127);
    delete h;
}

size_t ws_ints(int M) { return abft::ws_base_ints(M); }

}  // namespace

namespace abft {
int set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace abft

extern "C" {

const char* abft_last_error(void) { return g_err; }

int abft_pack_b_checksum(const int8_t* B, int64_t ldb, int K, int N, int b_is_transposed, void* stream,
                         abft_packed_b** out) {
    if (!B || !out) return fail(ABFT_EINVAL, "abft_pack_b_checksum: null pointer");
    if (K < 1 || N < 1) return fail(ABFT_EINVAL, "abft_pack_b_checksum: K=%d N=%d must be >= 1", K, N);
    if (ldb < (b_is_transposed ? K : N))
        return fail(ABFT_EINVAL, "abft_pack_b_checksum: ldb=%lld smaller than the row length", (long long)ldb);
    if (N > (1 << 23)) return fail(ABFT_EUNSUPPORTED, "abft_pack_b_checksum: N=%d above 2^23", N);
    abft_packed_b* h = new (std::nothrow) abft_packed_b();
    if (!h) return fail(ABFT_EHIP, "abft_pack_b_checksum: out of host memory");
    std::memset(h, 0, sizeof *h);
    h->K = K;
    h->N = N;
    h->KB = ((K + 2 * abft::kUnitK - 1) / (2 * abft::kUnitK)) * 2;
    h->NT = (N + abft::kTileN - 1) / abft::kTileN;
    hipError_t e = hipGetDevice(&h->device);
    const size_t packed_bytes = (size_t)h->NT * h->KB * abft::kUnitsPerTile * abft::kUnitBytes;
    if (e == hipSuccess) e = hipMalloc(&h->packed, packed_bytes);
    if (e == hipSuccess) e = hipMalloc(&h->limbs, (size_t)h->KB * abft::kUnitK * abft::kLimbs);
    if (e == hipSuccess) e = hipMalloc(&h->S_B, (size_t)h->KB * abft::kUnitK * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(&h->colsum, (size_t)h->NT * abft::kTileN * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(&h->total, 64);
    if (e == hipSuccess) e = hipMalloc(&h->limbs127, (size_t)h->KB * abft::kUnitK * abft::kLimbs);
    if (e == hipSuccess) e = hipMalloc(&h->S_B127, (size_t)h->KB * abft::kUnitK * sizeof(int32_t));
    if (e == hipSuccess) e = abft::launch_pack(B, ldb, b_is_transposed ? 1 : 0, h, (hipStream_t)stream);
    if (e != hipSuccess) {
        free_handle(h);
        return hip_fail(e, "abft_pack_b_checksum");
    }
    *out = h;
    return ABFT_OK;
}

int abft_packed_b_dims(const abft_packed_b* Bp, int* K, int* N) {
    if (!Bp) return fail(ABFT_EINVAL, "abft_packed_b_dims: null handle");
    if (K) *K = Bp->K;
    if (N) *N = Bp->N;
    return ABFT_OK;
}

int abft_packed_b_get_checksum(const abft_packed_b* Bp, int32_t* S_B, void* stream) {
    if (!Bp || !S_B) return fail(ABFT_EINVAL, "abft_packed_b_get_checksum: null pointer");
    HIP_TRY(hipMemcpyAsync(S_B, Bp->S_B, (size_t)Bp->K * sizeof(int32_t), hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_packed_b_get_checksum_mod127(const abft_packed_b* Bp, int32_t* rowSum, void* stream) {
    if (!Bp || !rowSum) return fail(ABFT_EINVAL, "abft_packed_b_get_checksum_mod127: null pointer");
    HIP_TRY(hipMemcpyAsync(rowSum, Bp->S_B127, (size_t)Bp->K * sizeof(int32_t), hipMemcpyDeviceToDevice,
                           (hipStream_t)stream));
    return ABFT_OK;
}

int abft_packed_b_get_col_offsets(const abft_packed_b* Bp, int32_t* colsum, void* stream) {
    if (!Bp || !colsum) return fail(ABFT_EINVAL, "abft_packed_b_get_col_offsets: null pointer");
    HIP_TRY(hipMemcpyAsync(colsum, Bp->colsum, (size_t)Bp->N * sizeof(int32_t), hipMemcpyDeviceToDevice,
                           (hipStream_t)stream));
    return ABFT_OK;
}

int abft_packed_b_flip_bit(abft_packed_b* Bp, int k, int j, int bit, void* stream) {
    if (!Bp) return fail(ABFT_EINVAL, "abft_packed_b_flip_bit: null handle");
    if (k < 0 || k >= Bp->K || j < 0 || j >= Bp->N || bit < 0 || bit > 7)
        return fail(ABFT_EINVAL, "abft_packed_b_flip_bit: (k=%d, j=%d, bit=%d) outside %dx%d int8", k, j, bit, Bp->K, Bp->N);
    HIP_TRY(abft::launch_flip_bit(Bp, k, j, bit, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_packed_b_flip_checksum_bit(abft_packed_b* Bp, int k, int bit, void* stream) {
    if (!Bp) return fail(ABFT_EINVAL, "abft_packed_b_flip_checksum_bit: null handle");
    if (k < 0 || k >= Bp->K || bit < 0 || bit > 31)
        return fail(ABFT_EINVAL, "abft_packed_b_flip_checksum_bit: (k=%d, bit=%d) outside [0,%d) x [0,32)", k, bit, Bp->K);
    HIP_TRY(abft::launch_flip_checksum_bit(Bp, k, bit, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_packed_b_flip_checksum_bit_mod127(abft_packed_b* Bp, int k, int bit, void* stream) {
    if (!Bp) return fail(ABFT_EINVAL, "abft_packed_b_flip_checksum_bit_mod127: null handle");
    if (k < 0 || k >= Bp->K || bit < 0 || bit > 7)
        return fail(ABFT_EINVAL, "abft_packed_b_flip_checksum_bit_mod127: (k=%d, bit=%d) outside [0,%d) x [0,8)", k, bit, Bp->K);
    HIP_TRY(abft::launch_flip_checksum127_bit(Bp, k, bit, (hipStream_t)stream));
    return ABFT_OK;
}

void abft_packed_b_destroy(abft_packed_b* Bp) { free_handle(Bp); }

size_t abft_gemm_workspace_bytes(int M, const abft_packed_b* Bp) {
    if (M < 1) return 0;
    // with the weight known: room for the partial tiles of a K split across workgroups, where one would be used
    if (Bp) return abft::splitk_plan(M, Bp->N, Bp->KB / 2).total_ints * sizeof(int32_t);
    return ws_ints(M) * sizeof(int32_t);
}

int abft_workspace_init(void* workspace, size_t bytes, void* stream) {
    if (!workspace && bytes) return fail(ABFT_EINVAL, "abft_workspace_init: null workspace");
    if (bytes % 4) return fail(ABFT_EINVAL, "abft_workspace_init: size must be a multiple of 4");
    HIP_TRY(abft::launch_fill_zero((int32_t*)workspace, bytes / 4, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_gemm_u8s8s32_checked(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp, int32_t* C,
                              int64_t ldc, int32_t* row_flags, int32_t* err_count, const abft_requant_t* rq,
                              uint8_t* Cq, int64_t ldcq, const abft_inject_t* inj, int n_inj, uint32_t flags,
                              void* workspace, size_t workspace_bytes, void* stream) {
    const char* fn = "abft_gemm_u8s8s32_checked";
    if (!A || !Bp) return fail(ABFT_EINVAL, "%s: null A or packed B", fn);
    if (M < 1) return fail(ABFT_EINVAL, "%s: M=%d must be >= 1", fn, M);
    if (lda < Bp->K) return fail(ABFT_EINVAL, "%s: lda=%lld < K=%d", fn, (long long)lda, Bp->K);
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != Bp->device)
        return fail(ABFT_EINVAL, "%s: the packed B lives on device %d, the current device is %d", fn, Bp->device, dev);
    const bool check = !(flags & ABFT_NOCHECK);
    const bool want_c = C != nullptr, want_q = rq != nullptr;
    if (!want_c && !want_q) return fail(ABFT_EINVAL, "%s: C is NULL and no requantization was asked for", fn);
    if (want_c && ldc < Bp->N) return fail(ABFT_EINVAL, "%s: ldc=%lld < N=%d", fn, (long long)ldc, Bp->N);
    if (want_q) {
        if (!Cq) return fail(ABFT_EINVAL, "%s: requantization asked for but Cq is NULL", fn);
        if (ldcq < Bp->N) return fail(ABFT_EINVAL, "%s: ldcq=%lld < N=%d", fn, (long long)ldcq, Bp->N);
        if (!rq->mult) return fail(ABFT_EINVAL, "%s: requantization multiplier is NULL", fn);
    }
    if (n_inj < 0 || (n_inj > 0 && !inj)) return fail(ABFT_EINVAL, "%s: bad injection list", fn);
    if (check) {
        if (!row_flags) return fail(ABFT_EINVAL, "%s: row_flags is NULL", fn);
        // (the row words are what a checked launch needs; the room for a K split across workgroups that
        // abft_gemm_workspace_bytes adds is optional: without it the launch runs unsplit)
        if (!workspace || workspace_bytes < ws_ints(M) * sizeof(int32_t))
            return fail(ABFT_EINVAL, "%s: workspace of %zu bytes, %zu needed", fn, workspace_bytes,
                        ws_ints(M) * sizeof(int32_t));
    }

    abft::GemmParams p;
    std::memset(&p, 0, sizeof p);
    p.A = A;
    p.lda = lda;
    p.M = M;
    p.N = Bp->N;
    p.K = Bp->K;
    p.KB = Bp->KB;
    p.KB2 = Bp->KB / 2;
    p.a_vec_ok = (((uintptr_t)A | (uintptr_t)lda) & 15) == 0;
    p.packed = Bp->packed;
    p.limbs = Bp->limbs;
    p.colsum = Bp->colsum;
    p.total = Bp->total;
    p.C = C;
    p.ldc = ldc;
    p.row_flags = row_flags;
    p.err_count = err_count;
    p.Cq = Cq;
    p.ldcq = ldcq;
    if (want_q) {
        p.rq.zA = rq->zA;
        p.rq.zC = rq->zC;
        p.rq.mult = rq->mult;
        p.rq.per_channel = rq->per_channel;
        p.rq.bias = rq->bias;
    }
    p.inj = inj;
    p.n_inj = n_inj;
    p.ws = (int32_t*)workspace;
    p.ws_ints = workspace ? workspace_bytes / sizeof(int32_t) : 0;
    p.ksplit = 1;
    p.err_accumulate = (flags & ABFT_ERRCOUNT_ACCUMULATE) != 0;
#ifdef ABFT_CLOCK_TRACE
    p.clock_trace = g_clock_trace.load(std::memory_order_acquire);
#endif
    const bool mod127 = check && (flags & ABFT_MOD127) != 0;
    if (mod127) {
        // exact (unwrapped) 32-bit entries are what the congruence modulo 127 needs
        if (Bp->K > 65536) return fail(ABFT_EUNSUPPORTED, "%s: modulus 127 needs K <= 65536, got %d", fn, Bp->K);
        p.mod127 = 1;
        p.limbs = Bp->limbs127;
        p.total = Bp->total + 1;
    }

    int variant = (int)((flags & ABFT_VARIANT_MASK) >> 8);
    const bool chosen = variant != 0;
    auto pick_tile = [&]() {
        // The larger the tile the better the matrix cores are fed, but a grid that leaves most of the
        // 256 compute units without a workgroup loses more than that: thresholds from timing the
        // three tile shapes on shapes between 128x2048 and 4096x4096.
        auto tiles = [&](int b) { return (int64_t)((M + b - 1) / b) * ((Bp->N + b - 1) / b); };
        if (tiles(256) >= 128) return (int)abft::kTile256;
        if (tiles(128) >= 136) return (int)abft::kTile128;  // (1024x2048x2048: 13.4 us on 64x64 tiles, 14.5 on 128x128)
        return (int)abft::kTile64;
    };
    // The streaming kernel reads the weight once and wins wherever that dominates: up to 32 rows always,
    // up to 64 rows when the weight is large (measured: 64x4096x2048 9.5 us against 10.1 us tiled, but
    // 64x1024x1024 7.0 against 6.5 and 64x256x512 6.3 against 5.3).
    const bool streaming = M <= 32 || (M <= 64 && (int64_t)Bp->N * Bp->K >= (int64_t)1 << 22);
    if (!chosen) variant = streaming ? (int)abft::kSmallM : pick_tile();
    hipError_t e;
    if (variant == abft::kSmallM) {
        if (M > 64) return fail(ABFT_EUNSUPPORTED, "%s: the streaming variant takes M <= 64, got %d", fn, M);
        e = abft::launch_gemm_smallm(check, want_c, want_q, p, (hipStream_t)stream);
        if (e == hipErrorNotSupported && !chosen)  // unaligned A: the general tiled path takes it
            e = abft::launch_gemm_tile(pick_tile(), check, want_c, want_q, p, (hipStream_t)stream);
    } else if (variant >= abft::kTile256 && variant < abft::kVariantEnd) {
        e = abft::launch_gemm_tile(variant, check, want_c, want_q, p, (hipStream_t)stream);
    } else {
        return fail(ABFT_EINVAL, "%s: unknown variant %d", fn, variant);
    }
    if (e == hipErrorNotSupported) return fail(ABFT_EUNSUPPORTED, "%s: variant %d is not available", fn, variant);
    if (e != hipSuccess) return hip_fail(e, fn);
    return ABFT_OK;
}

// ---- the entry point for callers that cannot allocate -------------------------------------------
// Its workspace is this file-scope device array: every GPU the library runs on holds its own copy,
// at its own address, until the process ends.
#define ABFT_STATIC_WS_INTS (64 + 2 * ABFT_STATIC_WS_MAX_M)
static_assert(ABFT_STATIC_WS_MAX_M % 64 == 0 && ABFT_STATIC_WS_INTS >= 64 + 4224, "covers the streaming kernel's words too");
static __device__ __align__(256) int32_t scratch[ABFT_STATIC_WS_INTS];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<int32_t*> g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device ordinal

// Device address of this device's copy of `scratch` (the array's name is only a host-side stand-in
// for it); looked up once per device, with that device current.
int static_scratch(int dev, int32_t** out) {
    if (dev < 0 || dev >= kMaxDevices) return fail(ABFT_EUNSUPPORTED, "device ordinal %d above %d", dev, kMaxDevices - 1);
    int32_t* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        HIP_TRY(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(ABFT_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // (two threads may both look it up: same answer)
    }
    *out = ptr;
    return ABFT_OK;
}
}  // namespace

int abft_gemm_u8s8s32_checked_static(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp, int32_t* C,
                                     int64_t ldc, int32_t* row_flags, int32_t* err_count, const abft_requant_t* rq,
                                     uint8_t* Cq, int64_t ldcq, const abft_inject_t* inj, int n_inj, uint32_t flags,
                                     void* stream) {
    const char* fn = "abft_gemm_u8s8s32_checked_static";
    if (M > ABFT_STATIC_WS_MAX_M)
        return fail(ABFT_EUNSUPPORTED, "%s: M=%d above the %d rows the built-in workspace holds", fn, M, ABFT_STATIC_WS_MAX_M);
    if (M < 1) return fail(ABFT_EINVAL, "%s: M=%d must be >= 1", fn, M);
    if (flags & ABFT_NOCHECK)
        return abft_gemm_u8s8s32_checked(A, lda, M, Bp, C, ldc, row_flags, err_count, rq, Cq, ldcq, inj, n_inj, flags,
                                         nullptr, 0, stream);
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    int32_t* ws = nullptr;
    const int rc = static_scratch(dev, &ws);
    if (rc != ABFT_OK) return rc;
    const size_t ints = ws_ints(M);
    // the array keeps whatever the last call on this device left (zeros, unless that call was cut short):
    // the words this call counts on start at zero (a fill kernel, so that the call may be captured in a graph)
    HIP_TRY(abft::launch_fill_zero(ws, ints, (hipStream_t)stream));
    return abft_gemm_u8s8s32_checked(A, lda, M, Bp, C, ldc, row_flags, err_count, rq, Cq, ldcq, inj, n_inj, flags, ws,
                                     ints * sizeof(int32_t), stream);
}

int abft_requantize_u8(const int32_t* C, int64_t ldc, int M, int N, const abft_packed_b* Bp,
                       const abft_requant_t* rq, uint8_t* Cq, int64_t ldcq, void* stream) {
    const char* fn = "abft_requantize_u8";
    if (!C || !Bp || !rq || !Cq || !rq->mult) return fail(ABFT_EINVAL, "%s: null pointer", fn);
    if (M < 1 || N < 1 || N != Bp->N) return fail(ABFT_EINVAL, "%s: M=%d N=%d (packed N=%d)", fn, M, N, Bp->N);
    if (ldc < N || ldcq < N) return fail(ABFT_EINVAL, "%s: leading dimension below N", fn);
    abft::RequantDev r{rq->zA, rq->zC, rq->mult, rq->per_channel, rq->bias};
    HIP_TRY(abft::launch_requantize(C, ldc, M, N, Bp->colsum, r, Cq, ldcq, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_verify_rows(const int32_t* C, int64_t ldc, int M, int N, const int32_t* row_chk, int32_t* row_flags,
                     int32_t* err_count, void* stream) {
    const char* fn = "abft_verify_rows";
    if (!C || !row_chk || !row_flags) return fail(ABFT_EINVAL, "%s: null pointer", fn);
    if (M < 1 || N < 1 || ldc < N) return fail(ABFT_EINVAL, "%s: M=%d N=%d ldc=%lld", fn, M, N, (long long)ldc);
    HIP_TRY(abft::launch_verify_rows(C, ldc, M, N, row_chk, row_flags, err_count, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_row_checksum(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp, int32_t* row_chk,
                      void* stream) {
    const char* fn = "abft_row_checksum";
    if (!A || !Bp || !row_chk) return fail(ABFT_EINVAL, "%s: null pointer", fn);
    if (M < 1 || lda < Bp->K) return fail(ABFT_EINVAL, "%s: M=%d lda=%lld K=%d", fn, M, (long long)lda, Bp->K);
    HIP_TRY(abft::launch_row_checksum(A, lda, M, Bp->K, Bp->S_B, row_chk, (hipStream_t)stream));
    return ABFT_OK;
}

namespace {
// layout of the recovery scratch for batches of `rows` rows against Bp
struct RecoverLayout {
    size_t idx, count, cnt2, flags2, a2, c2, q2, ws, total;
    int64_t lda2;
    size_t ws_bytes;
};
RecoverLayout recover_layout(int M, int rows, const abft_packed_b* Bp) {
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    RecoverLayout L;
    L.lda2 = ((int64_t)Bp->K + 15) / 16 * 16;
    L.ws_bytes = ws_ints(rows) * sizeof(int32_t);
    size_t o = 0;
    L.idx = o; o = up(o + (size_t)M * 4);
    L.count = o; o = up(o + 4);
    L.cnt2 = o; o = up(o + 4);
    L.flags2 = o; o = up(o + (size_t)rows * 4);
    L.a2 = o; o = up(o + (size_t)rows * L.lda2);
    L.c2 = o; o = up(o + (size_t)rows * Bp->N * 4);
    L.q2 = o; o = up(o + (size_t)rows * Bp->N);
    L.ws = o; o = up(o + L.ws_bytes);
    L.total = o;
    return L;
}
}  // namespace

size_t abft_recover_scratch_bytes(int M, int max_rows_per_pass, const abft_packed_b* Bp) {
    if (M < 1 || max_rows_per_pass < 1 || !Bp) return 0;
    return recover_layout(M, max_rows_per_pass, Bp).total;
}

int abft_recompute_flagged_rows(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp, int32_t* C, int64_t ldc,
                                int32_t* row_flags, int32_t* err_count, const abft_requant_t* rq, uint8_t* Cq,
                                int64_t ldcq, int max_rows_per_pass, void* scratch, size_t scratch_bytes, void* stream,
                                int* rows_before, int* rows_after) {
    const char* fn = "abft_recompute_flagged_rows";
    if (!A || !Bp || !row_flags || !scratch) return fail(ABFT_EINVAL, "%s: null pointer", fn);
    if (M < 1 || max_rows_per_pass < 1 || lda < Bp->K) return fail(ABFT_EINVAL, "%s: bad shape", fn);
    if (!C && !rq) return fail(ABFT_EINVAL, "%s: C is NULL and no requantization was asked for", fn);
    if ((C && ldc < Bp->N) || (rq && (!Cq || ldcq < Bp->N))) return fail(ABFT_EINVAL, "%s: bad output", fn);
    const RecoverLayout L = recover_layout(M, max_rows_per_pass, Bp);
    if (scratch_bytes < L.total) return fail(ABFT_EINVAL, "%s: scratch of %zu bytes, %zu needed", fn, scratch_bytes, L.total);
    hipStream_t s = (hipStream_t)stream;
    uint8_t* const base = (uint8_t*)scratch;
    int32_t* const idx = (int32_t*)(base + L.idx);
    int32_t* const count = (int32_t*)(base + L.count);
    int32_t* const cnt2 = (int32_t*)(base + L.cnt2);
    int32_t* const flags2 = (int32_t*)(base + L.flags2);
    uint8_t* const A2 = base + L.a2;
    int32_t* const C2 = (int32_t*)(base + L.c2);
    uint8_t* const Q2 = base + L.q2;
    HIP_TRY(abft::launch_list_flagged(row_flags, M, idx, count, s));
    int n = 0;
    HIP_TRY(hipMemcpyAsync(&n, count, sizeof n, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (rows_before) *rows_before = n;
    int remaining = 0;
    if (n > 0) {
        HIP_TRY(abft::launch_fill_zero((int32_t*)(base + L.ws), L.ws_bytes / 4, s));
        if (err_count) HIP_TRY(abft::launch_fill_zero(err_count, 1, s));
        for (int at = 0; at < n; at += max_rows_per_pass) {
            const int m = n - at < max_rows_per_pass ? n - at : max_rows_per_pass;
            HIP_TRY(abft::launch_gather_rows(A, lda, idx + at, m, Bp->K, A2, L.lda2, s));
            const int rc = abft_gemm_u8s8s32_checked(A2, L.lda2, m, Bp, C ? C2 : nullptr, Bp->N, flags2, cnt2, rq,
                                                     rq ? Q2 : nullptr, Bp->N, nullptr, 0, ABFT_CHECK, base + L.ws,
                                                     L.ws_bytes, stream);
            if (rc != ABFT_OK) return rc;
            HIP_TRY(abft::launch_scatter_rows(C ? C2 : nullptr, rq ? Q2 : nullptr, flags2, idx + at, m, Bp->N, C, ldc,
                                              rq ? Cq : nullptr, ldcq, row_flags, s));
            if (err_count) HIP_TRY(abft::launch_add_int(err_count, cnt2, s));
            if (rows_after) {
                int c = 0;
                HIP_TRY(hipMemcpyAsync(&c, cnt2, sizeof c, hipMemcpyDeviceToHost, s));
                HIP_TRY(hipStreamSynchronize(s));
                remaining += c;
            }
        }
    }
    if (rows_after) *rows_after = remaining;
    return ABFT_OK;
}

int abft_recompute_flagged_rows_async(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp, int32_t* C, int64_t ldc,
                                      int32_t* row_flags, int32_t* err_count, const abft_requant_t* rq, uint8_t* Cq,
                                      int64_t ldcq, int max_rows, void* scratch, size_t scratch_bytes, int32_t* status,
                                      void* stream) {
    const char* fn = "abft_recompute_flagged_rows_async";
    if (!A || !Bp || !row_flags || !scratch) return fail(ABFT_EINVAL, "%s: null pointer", fn);
    if (M < 1 || max_rows < 1 || lda < Bp->K) return fail(ABFT_EINVAL, "%s: bad shape", fn);
    if (!C && !rq) return fail(ABFT_EINVAL, "%s: C is NULL and no requantization was asked for", fn);
    if ((C && ldc < Bp->N) || (rq && (!Cq || ldcq < Bp->N))) return fail(ABFT_EINVAL, "%s: bad output", fn);
    const RecoverLayout L = recover_layout(M, max_rows, Bp);
    if (scratch_bytes < L.total) return fail(ABFT_EINVAL, "%s: scratch of %zu bytes, %zu needed", fn, scratch_bytes, L.total);
    hipStream_t s = (hipStream_t)stream;
    uint8_t* const base = (uint8_t*)scratch;
    int32_t* const idx = (int32_t*)(base + L.idx);
    int32_t* const count = (int32_t*)(base + L.count);
    int32_t* const cnt2 = (int32_t*)(base + L.cnt2);
    int32_t* const flags2 = (int32_t*)(base + L.flags2);
    uint8_t* const A2 = base + L.a2;
    int32_t* const C2 = (int32_t*)(base + L.c2);
    uint8_t* const Q2 = base + L.q2;
    HIP_TRY(abft::launch_list_flagged(row_flags, M, idx, count, s));
    HIP_TRY(abft::launch_gather_rows_bounded(A, lda, idx, count, max_rows, Bp->K, A2, L.lda2, s));
    HIP_TRY(abft::launch_fill_zero((int32_t*)(base + L.ws), L.ws_bytes / 4, s));
    const int rc = abft_gemm_u8s8s32_checked(A2, L.lda2, max_rows, Bp, C ? C2 : nullptr, Bp->N, flags2, cnt2, rq, rq ? Q2 : nullptr,
                                             Bp->N, nullptr, 0, ABFT_CHECK, base + L.ws, L.ws_bytes, stream);
    if (rc != ABFT_OK) return rc;
    HIP_TRY(abft::launch_scatter_rows_bounded(C ? C2 : nullptr, rq ? Q2 : nullptr, flags2, idx, count, max_rows, Bp->N, C, ldc,
                                              rq ? Cq : nullptr, ldcq, row_flags, s));
    HIP_TRY(abft::launch_recount(count, cnt2, max_rows, err_count, status, s));
    return ABFT_OK;
}

size_t abft_locate_scratch_bytes(const abft_packed_b* Bp) {
    if (!Bp) return 0;
    return ((size_t)Bp->KB * abft::kUnitK + 2 * (size_t)Bp->NT * abft::kTileN) * sizeof(int32_t);
}

int abft_locate_correct(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp, int32_t* C, int64_t ldc,
                        int32_t* row_flags, int32_t* err_count, const abft_requant_t* rq, uint8_t* Cq, int64_t ldcq,
                        int32_t* col_flags, abft_locate_t* report, void* scratch, size_t scratch_bytes, void* stream) {
    const char* fn = "abft_locate_correct";
    if (!A || !Bp || !C || !row_flags || !report || !scratch) return fail(ABFT_EINVAL, "%s: null pointer", fn);
    if (M < 1 || lda < Bp->K || ldc < Bp->N) return fail(ABFT_EINVAL, "%s: bad shape (M=%d lda=%lld ldc=%lld)", fn, M, (long long)lda, (long long)ldc);
    if (rq && (!Cq || ldcq < Bp->N || !rq->mult)) return fail(ABFT_EINVAL, "%s: bad requantized output", fn);
    if (scratch_bytes < abft_locate_scratch_bytes(Bp))
        return fail(ABFT_EINVAL, "%s: scratch of %zu bytes, %zu needed", fn, scratch_bytes, abft_locate_scratch_bytes(Bp));
    if (((uintptr_t)scratch | (uintptr_t)report) & 3) return fail(ABFT_EINVAL, "%s: scratch and report must be 4-byte aligned", fn);
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != Bp->device)
        return fail(ABFT_EINVAL, "%s: the packed B lives on device %d, the current device is %d", fn, Bp->device, dev);
    abft::RequantDev r{};
    if (rq) r = abft::RequantDev{rq->zA, rq->zC, rq->mult, rq->per_channel, rq->bias};
    HIP_TRY(abft::launch_locate_correct(A, lda, M, Bp, C, ldc, row_flags, err_count, rq ? &r : nullptr, Cq, ldcq, col_flags,
                                        reinterpret_cast<int32_t*>(report), (int32_t*)scratch, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_calib_copy(const void* src, void* dst, size_t bytes, void* stream) {
    const char* fn = "abft_calib_copy";
    if (!src || !dst) return fail(ABFT_EINVAL, "%s: null pointer", fn);
    if (bytes == 0 || bytes % 16 != 0 || ((uintptr_t)src | (uintptr_t)dst) % 16 != 0)
        return fail(ABFT_EINVAL, "%s: bytes=%zu and both pointers must be multiples of 16", fn, bytes);
    HIP_TRY(abft::launch_calib_copy(src, dst, bytes, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_clock_probe(uint64_t* out, int microseconds, void* stream) {
    const char* fn = "abft_clock_probe";
    if (!out || ((uintptr_t)out & 7)) return fail(ABFT_EINVAL, "%s: out must be an 8-byte aligned device pointer", fn);
    if (microseconds < 1 || microseconds > 100000) return fail(ABFT_EINVAL, "%s: %d us outside [1, 100000]", fn, microseconds);
    HIP_TRY(abft::launch_clock_probe(reinterpret_cast<unsigned long long*>(out), 100ull * (unsigned long long)microseconds,
                                     (hipStream_t)stream));
    return ABFT_OK;
}

int abft_mfma_peak_probe(uint64_t* out, int iters, void* stream) {
    const char* fn = "abft_mfma_peak_probe";
    if (!out || ((uintptr_t)out & 7)) return fail(ABFT_EINVAL, "%s: out must be an 8-byte aligned device pointer", fn);
    if (iters < 1 || iters > (1 << 22)) return fail(ABFT_EINVAL, "%s: iters=%d outside [1, 2^22]", fn, iters);
    HIP_TRY(abft::launch_mfma_peak_probe(reinterpret_cast<unsigned long long*>(out), iters, (hipStream_t)stream));
    return ABFT_OK;
}

int abft_clock_trace(uint64_t* buf) {
#ifdef ABFT_CLOCK_TRACE
    g_clock_trace.store(reinterpret_cast<unsigned long long*>(buf), std::memory_order_release);
    return ABFT_OK;
#else
    (void)buf;
    return fail(ABFT_EUNSUPPORTED, "abft_clock_trace: this library was built without ABFT_CLOCK_TRACE "
                                   "(python -m paper_2103_00130_amd.build --clock-trace builds the diagnostic library)");
#endif
}

}  // extern "C"
