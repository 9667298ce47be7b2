/*
 * libabftgemm: ABFT-checked u8 x s8 -> s32 GEMM for AMD MI355X (gfx950).
 *
 * The operation is Algorithm 1 of arXiv 2103.00130 ("ABFT for low-precision
 * GEMM", Section IV) on the quantized product of Section III (Eq. 1): the
 * weight matrix B is encoded once with its checksum column S_B = B e
 * (Section IV-A-1: only B is encoded), the checksum is packed together with B
 * (Section IV-A-3) so that C_temp = A * [B | S_B] comes out of one pass, and
 * every row of the 32-bit intermediate is verified with the row identity of
 * Eq. 2b before requantization (Section IV-B).  One deliberate difference from
 * the printed algorithm: the checksum column is kept exact (int32, carried
 * through the int8 matrix cores as four signed base-256 digits) and the
 * comparison is an equality of wrap-around int32 values (mod 2^32) rather
 * than mod 127.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer owned by the caller unless a comment
 *     says "host".  Matrices are row-major with a leading dimension in
 *     elements.  `stream` is a hipStream_t passed as void* (NULL = default
 *     stream).  Calls enqueue work on `stream` and return; they never
 *     synchronise.  Only abft_pack_b_checksum / abft_packed_b_destroy
 *     allocate or free device memory.  A packed B belongs to the device that
 *     was current when it was packed; the checked GEMM returns ABFT_EINVAL
 *     when called with another device current.
 *   - Return value: ABFT_OK, or a negative code for a usage or runtime error;
 *     abft_last_error() then gives a message (thread-local, host).  Nothing is
 *     enqueued when a call returns ABFT_EINVAL or ABFT_EUNSUPPORTED.
 *   - A DETECTED SOFT ERROR IS NOT AN ERROR RETURN.  It is data: row_flags and
 *     err_count, the "number of corrupted rows" output of Algorithm 1.
 *   - B is symmetric-quantized (zero point 0): the row-offset term
 *     alpha_A beta_B (A_I e_k) e_n^T of Eq. 1 is not part of this library.
 */
#ifndef ABFT_GEMM_H
#define ABFT_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ABFT_OK 0
#define ABFT_EINVAL (-1)        /* null pointer, bad shape, ld < dim, workspace too small */
#define ABFT_EUNSUPPORTED (-2)  /* valid request this build does not implement */
#define ABFT_EHIP (-3)          /* a HIP runtime call failed */

/* flags of abft_gemm_u8s8s32_checked */
#define ABFT_CHECK 0u             /* default: verify every row (Algorithm 1) */
#define ABFT_NOCHECK 1u           /* same kernel with the checksum work compiled out */
#define ABFT_MOD127 2u            /* Algorithm 1 to the letter: the checksum column is
                                     rowSum = (B e) mod 127, one 8-bit column (Section
                                     IV-A-2), and a row is flagged when its sum and its
                                     checksum entry differ modulo 127.  16-byte aligned
                                     A with K a multiple of 16, K <= 65536. */
#define ABFT_ERRCOUNT_ACCUMULATE 4u /* errCount as Algorithm 1 writes it, a counter that is
                                     incremented: the number of flagged rows is ADDED to
                                     *err_count (which the caller set, normally to zero, and
                                     may leave to run over several calls) instead of
                                     overwriting it.  A launch that flags nothing does not
                                     touch the counter, and no workgroup has to learn that
                                     it is the last one, which takes one dependent memory
                                     round trip off the end of every launch. */
#define ABFT_VARIANT_MASK 0xF00u  /* 0 = choose by shape */
#define ABFT_VARIANT_TILE256 0x100u
#define ABFT_VARIANT_TILE128 0x200u
#define ABFT_VARIANT_TILE64 0x300u
#define ABFT_VARIANT_SMALLM 0x400u /* streaming kernel, M <= 64 */
#define ABFT_VARIANT_TILE256_W2X4 0x500u /* 256x256 tile, 8 wavefronts as 2x4 */
#define ABFT_VARIANT_TILE256_W4X2 0x600u /* 256x256 tile, 8 wavefronts as 4x2 */

/* Opaque packed weight: B in matrix-core fragment order, its checksum column
 * S_B = B e as four signed base-256 digit columns, S_B itself, and the column
 * sums e^T B used by the zero-point correction of Eq. 1.  The library owns
 * its device memory. */
typedef struct abft_packed_b abft_packed_b;

/* Algorithm 1, the encode and pack steps (rowSum[] loop and pack(B, rowSum[])),
 * done once per weight matrix (Section IV-A-1: the cost is amortised).
 *   B    int8, K x N row-major with ldb >= N when b_is_transposed == 0;
 *        N x K row-major with ldb >= K (a torch Linear weight) when 1.
 *   out  host pointer receiving the handle.
 * Allocates with hipMalloc; the packing kernels are enqueued on `stream`, and
 * B must stay valid until they have run. */
int abft_pack_b_checksum(const int8_t* B, int64_t ldb, int K, int N, int b_is_transposed,
                         void* stream, abft_packed_b** out);

/* K and N of a packed weight (host out-pointers, either may be NULL). */
int abft_packed_b_dims(const abft_packed_b* Bp, int* K, int* N);

/* Copy S_B = B e (int32 [K]; Section IV, definition of the encoded column). */
int abft_packed_b_get_checksum(const abft_packed_b* Bp, int32_t* S_B, void* stream);

/* rowSum[k] = (B e)[k] mod 127 in [0,126] as int32 [K]: the 8-bit checksum column
 * of Algorithm 1 as printed, for parity checks of ABFT_MOD127. */
int abft_packed_b_get_checksum_mod127(const abft_packed_b* Bp, int32_t* rowSum, void* stream);

/* Copy e^T B (int32 [N]; rank-1 term of Eq. 1). */
int abft_packed_b_get_col_offsets(const abft_packed_b* Bp, int32_t* colsum, void* stream);

/* Fault-injection hooks (the fault model of Section VI-B: one bit of one
 * randomly chosen element is inverted, in B after its checksum was computed).
 * flip_bit inverts bit `bit` (0..7) of logical B[k][j] inside the packed
 * layout and leaves the checksum stale; flip_checksum_bit inverts bit `bit`
 * (0..31) of the stored checksum entry S_B[k] as the kernels see it (the paper
 * assumes this column error-free, Section IV-C).  Calling either twice with
 * the same arguments restores the weight. */
int abft_packed_b_flip_bit(abft_packed_b* Bp, int k, int j, int bit, void* stream);
int abft_packed_b_flip_checksum_bit(abft_packed_b* Bp, int k, int bit, void* stream);
/* The same hook for the 8-bit column that ABFT_MOD127 reads (Section IV-A-2):
 * inverts bit `bit` (0..7) of the stored int8 rowSum[k].  flip_checksum_bit above
 * touches only the int32 column of the default check, this one only the 8-bit
 * column; abft_packed_b_get_checksum_mod127 returns the entry as it now stands
 * (sign-extended when bit 7 was inverted). */
int abft_packed_b_flip_checksum_bit_mod127(abft_packed_b* Bp, int k, int bit, void* stream);

/* Host call.  Frees the handle; the caller has synchronised every stream that
 * used it. */
void abft_packed_b_destroy(abft_packed_b* Bp);

/* Requantization parameters (Section III-B; Eq. 1 with beta_B = 0):
 *   t = C_temp[i][j] - zA * colsum_B[j] (+ bias[j]);  y = clamp(rne(float(t) * mult) + zC, 0, 255)
 * in binary32 with round-to-nearest-even.  HOST struct; `mult` (1 value, or N
 * when per_channel) and `bias` (N, or NULL) are device pointers. */
typedef struct {
    int32_t zA;
    int32_t zC;
    const float* mult;
    int32_t per_channel;
    const int32_t* bias;
} abft_requant_t;

/* One simulated fault in the 32-bit intermediate (the fault model of Section
 * VI-B-1, a bit flip in the 32-bit result matrix): C_temp[row][col] ^= xor_mask
 * after the product and before the row sums, the store and the
 * requantization.  Entries that name the same element act as one entry with
 * the XOR of their masks; entries outside the M x N matrix are ignored. */
typedef struct {
    int32_t row;
    int32_t col;
    uint32_t xor_mask;
} abft_inject_t;

/* Scratch the checked GEMM needs for a problem with M rows against Bp: one
 * 64-bit word per row (partial row sum - checksum, and how many column blocks
 * have contributed) and a few counting words (rows finished, rows corrupted);
 * with Bp given, also room for the partial tiles of a K split across
 * workgroups on the shapes where the library uses one (few tiles, K of about
 * 5000 and more; Bp == NULL, or a smaller workspace of at least the size this
 * call returns for Bp == NULL, runs every shape unsplit).
 * The memory must be zero before its first use (abft_workspace_init) and every
 * call leaves it zero again, so one workspace serves any number of calls that
 * are ordered on one stream.  Calls that may overlap need one workspace each. */
size_t abft_gemm_workspace_bytes(int M, const abft_packed_b* Bp);
int abft_workspace_init(void* workspace, size_t bytes, void* stream);

/* Algorithm 1 from the product line to the return: C_temp = A * [B | S_B] in
 * one pass over A, tSum per row, comparison (Eq. 2b, equality mod 2^32),
 * errCount; optionally the requantization that follows it (Section IV-B: the
 * check reads the 32-bit values, requantization excludes the checksum column).
 *   A          uint8 M x K row-major, lda >= K.  Fast path when A and lda are
 *              multiples of 16 bytes; any alignment is accepted.
 *   C          int32 M x N, ldc >= N; may be NULL when rq != NULL (then only
 *              the uint8 output is written).
 *   row_flags  int32 [M], overwritten with 0/1 per row (ignored with ABFT_NOCHECK).
 *   err_count  int32 [1], overwritten with the number of flagged rows (added to
 *              with ABFT_ERRCOUNT_ACCUMULATE); may be NULL.
 *   rq, Cq     host struct or NULL; uint8 M x N output with ldcq >= N.
 *   inj        device array of n_inj simulated faults, or NULL / 0.
 *   flags      ABFT_CHECK or ABFT_NOCHECK, optionally | ABFT_MOD127,
 *              | ABFT_ERRCOUNT_ACCUMULATE, | ABFT_VARIANT_*.
 *   workspace  abft_gemm_workspace_bytes(M, Bp) bytes, zeroed once; may be
 *              NULL with ABFT_NOCHECK.
 * Errors: ABFT_EINVAL for null/shape/ld/workspace problems (inj is device
 * memory and is not inspected on the host); ABFT_EUNSUPPORTED for a variant
 * that cannot run the shape; ABFT_EHIP for a failed launch. */
int abft_gemm_u8s8s32_checked(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp,
                              int32_t* C, int64_t ldc, int32_t* row_flags, int32_t* err_count,
                              const abft_requant_t* rq, uint8_t* Cq, int64_t ldcq,
                              const abft_inject_t* inj, int n_inj, uint32_t flags,
                              void* workspace, size_t workspace_bytes, void* stream);

/* abft_gemm_u8s8s32_checked for callers that cannot allocate device memory and
 * have no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same
 * kernels, same results; the counting words live in a device array built into
 * the library (one copy per GPU, ABFT_STATIC_WS_MAX_M rows at most, about 1 MiB,
 * held until the process ends).  The call itself allocates nothing and frees
 * nothing; it enqueues one small fill kernel that zeroes the words it is about
 * to use, then the GEMM.  Every call on one GPU shares that GPU's array: calls
 * that may overlap on one GPU (different streams, no ordering) race - order them
 * or use abft_gemm_u8s8s32_checked with one workspace per stream.
 * Errors: as abft_gemm_u8s8s32_checked; ABFT_EUNSUPPORTED when
 * M > ABFT_STATIC_WS_MAX_M. */
#define ABFT_STATIC_WS_MAX_M 131072
int abft_gemm_u8s8s32_checked_static(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp,
                                     int32_t* C, int64_t ldc, int32_t* row_flags, int32_t* err_count,
                                     const abft_requant_t* rq, uint8_t* Cq, int64_t ldcq,
                                     const abft_inject_t* inj, int n_inj, uint32_t flags, void* stream);

/* Stand-alone requantization of a stored int32 C_temp (Section III-B), using the
 * column sums held in Bp.  Same arithmetic as the fused epilogue. */
int abft_requantize_u8(const int32_t* C, int64_t ldc, int M, int N, const abft_packed_b* Bp,
                       const abft_requant_t* rq, uint8_t* Cq, int64_t ldcq, void* stream);

/* Re-verification of a C_temp that has been sitting in memory (the paper's
 * "flip in the 32-bit intermediate" fault model applied after the GEMM):
 * row_chk[i] = (A S_B)[i] as produced by abft_row_checksum, or supplied by the
 * caller; flags rows whose sum differs.  */
int abft_verify_rows(const int32_t* C, int64_t ldc, int M, int N, const int32_t* row_chk,
                     int32_t* row_flags, int32_t* err_count, void* stream);

/* chk = A S_B (int32 [M]) on its own, from A and the packed checksum digits:
 * the reference side of Eq. 2b for abft_verify_rows. */
int abft_row_checksum(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp,
                      int32_t* row_chk, void* stream);

/* What the method does once a row is flagged: recompute it (Section I: on
 * detection the affected result is recomputed; Section IV keeps the scheme to
 * detection so that this is the only recovery).  The rows whose flag is set are
 * gathered from A, multiplied and checked again in passes of at most
 * max_rows_per_pass rows, and written back into C / Cq; row_flags and err_count
 * are updated to the verdicts of the recomputation, so a transient fault leaves
 * them at zero and a fault that persists in memory (in B, say) leaves them set.
 * UNLIKE EVERY OTHER CALL THIS ONE SYNCHRONISES `stream`: the number of flagged
 * rows has to reach the host.  rows_before / rows_after (host, may be NULL)
 * receive the number of flagged rows found and the number still flagged.
 * scratch: device memory of abft_recover_scratch_bytes(M, max_rows_per_pass, Bp)
 * bytes, contents irrelevant.  A, lda, rq as for abft_gemm_u8s8s32_checked. */
size_t abft_recover_scratch_bytes(int M, int max_rows_per_pass, const abft_packed_b* Bp);
int abft_recompute_flagged_rows(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp,
                                int32_t* C, int64_t ldc, int32_t* row_flags, int32_t* err_count,
                                const abft_requant_t* rq, uint8_t* Cq, int64_t ldcq,
                                int max_rows_per_pass, void* scratch, size_t scratch_bytes, void* stream,
                                int* rows_before, int* rows_after);

/* The same recovery without a round trip to the host: the number of flagged
 * rows stays on the device and bounds the gather and scatter kernels there, so
 * the call only enqueues work (six small launches around one checked GEMM of
 * max_rows rows) and returns.  At most max_rows flagged rows are recomputed in
 * the one pass (any others keep their flag; soft errors are rare, one row is the
 * expected case, and max_rows <= 64 keeps the recomputation on the streaming
 * kernel: one pass over the weight).
 *   status   DEVICE int32 [2], may be NULL: [0] flagged rows found, [1] rows still
 *            flagged afterwards (also written to *err_count when that is given).
 *   scratch  abft_recover_scratch_bytes(M, max_rows, Bp) bytes. */
int abft_recompute_flagged_rows_async(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp,
                                      int32_t* C, int64_t ldc, int32_t* row_flags, int32_t* err_count,
                                      const abft_requant_t* rq, uint8_t* Cq, int64_t ldcq, int max_rows,
                                      void* scratch, size_t scratch_bytes, int32_t* status, void* stream);

/* Locating and correcting one faulty element of C_temp (Section IV: the column
 * check of Eq. 2a next to the row check of Eq. 2b, and the two correction
 * formulas that follow them).  The product itself stays with detection and an
 * encoded B only, as the paper prescribes (Section IV-A-1); this call is the
 * other half of the classic scheme, run on demand once a launch has flagged
 * something: it forms S_A = e^T A from the A in memory, the checksum row
 * C'[m][:] = S_A B from the packed weight, and the column sums of the stored
 * C_temp (all wrap-around int32).  When exactly one row is flagged in row_flags
 * (the verdicts of Eq. 2b as abft_gemm_u8s8s32_checked returned them) and exactly
 * one column violates Eq. 2a, the element where they cross is recomputed as
 *     C'[m][j] - sum_{p != i} C[p][j]
 * and, as a cross-check, as (A S_B)[i] - sum_{p != j} C[i][p]; if the two agree the
 * value is written to C (and requantized into Cq when rq != NULL), row_flags[i]
 * is cleared and *err_count is decremented.  Any other pattern - several rows or
 * columns, rows without a column (a fault in B after it was encoded corrupts a
 * column of C consistently with the B in memory), formulas that disagree - leaves
 * C, row_flags and err_count as they are.
 *   A, lda, M, Bp, C, ldc, rq, Cq, ldcq   as for abft_gemm_u8s8s32_checked (C must
 *              be present: the check reads the stored 32-bit values).
 *   col_flags  int32 [N], overwritten with the verdicts of Eq. 2a; may be NULL.
 *   report     DEVICE memory for one abft_locate_t, overwritten.
 *   scratch    abft_locate_scratch_bytes(Bp) bytes of device memory, contents
 *              irrelevant.
 * Asynchronous like every other call; four small kernels, about one pass over A,
 * the packed B and C. */
#define ABFT_LOCATE_CLEAN 0            /* no row flagged, no column violated */
#define ABFT_LOCATE_CORRECTED 1        /* one element located and rewritten */
#define ABFT_LOCATE_NOT_ONE_ELEMENT 2  /* violations that do not single out one element; nothing written */
typedef struct {
    int32_t status;        /* ABFT_LOCATE_* */
    int32_t row, col;      /* the element (status CORRECTED), else -1 */
    int32_t old_value;     /* what was stored there */
    int32_t new_value;     /* what was written */
    int32_t rows_flagged;  /* rows set in row_flags on entry */
    int32_t cols_violated; /* columns violating Eq. 2a */
    int32_t reserved;
} abft_locate_t;
size_t abft_locate_scratch_bytes(const abft_packed_b* Bp);
int abft_locate_correct(const uint8_t* A, int64_t lda, int M, const abft_packed_b* Bp, int32_t* C, int64_t ldc,
                        int32_t* row_flags, int32_t* err_count, const abft_requant_t* rq, uint8_t* Cq,
                        int64_t ldcq, int32_t* col_flags, abft_locate_t* report, void* scratch,
                        size_t scratch_bytes, void* stream);

/* Measurement aid, not part of the method: a plain device-to-device copy of
 * `bytes` (a positive multiple of 16; both pointers 16-byte aligned, buffers
 * must not overlap).  It reads and writes exactly `bytes` once, which makes it
 * the known-size reference that a profiler's HBM traffic counters are scaled
 * by when the GEMM kernels' traffic is reported. */
int abft_calib_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Measurement aid, not part of the method: one lane samples the shader-clock
 * cycle counter and the constant 100 MHz wall counter, waits `microseconds`
 * (1..100000) of wall time, and samples both again.  out (DEVICE, 4 x uint64):
 * wall ticks and shader cycles at the start, wall ticks and shader cycles at
 * the end; (cycles end - start) / (ticks end - start) x 100 MHz is the shader
 * clock in that interval.  Enqueued on a stream of its own next to a run of
 * GEMM launches it shows the clock the chip sustains under that load, which is
 * what the matrix-core roofline has to be read against. */
int abft_clock_probe(uint64_t* out, int microseconds, void* stream);

/* Measurement aid: a register-only matrix-core load.  256 workgroups of four
 * wavefronts run `iters` rounds of four independent 32x32x32 int8 MFMAs on
 * operands that stay in registers; out (DEVICE, 4 x uint64 per workgroup, 256
 * workgroups): shader cycles and 100 MHz wall ticks before and after the loop.
 * 256 x 4 x iters x 4 x 65536 operations over the wall time is what the matrix
 * cores deliver, and cycles over wall time the clock they hold, when neither
 * LDS nor memory draws power: the reference the GEMM's in-loop figures are read
 * against. */
int abft_mfma_peak_probe(uint64_t* out, int iters, void* stream);

/* Diagnostic builds only (the library compiled with ABFT_CLOCK_TRACE, see
 * build.py --clock-trace; ABFT_EUNSUPPORTED otherwise): from now on every
 * direct-to-LDS tiled launch writes, per workgroup, 6 x uint64 to buf (DEVICE,
 * sized for the largest grid the caller launches; NULL switches it off):
 * shader cycles and 100 MHz wall ticks before the K loop, after it, and at the
 * end of the kernel.  Process-wide; the product library carries no such code. */
int abft_clock_trace(uint64_t* buf);

/* Message for the last non-OK return on this host thread. */
const char* abft_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ABFT_GEMM_H */
