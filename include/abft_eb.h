/*
 * libabftgemm, second operator: ABFT-checked low-precision EmbeddingBag for AMD MI355X
 * (gfx950).
 *
 * The operation is Algorithm 2 of arXiv 2103.00130 ("ABFT for low-precision EB",
 * Section V) on the row-wise quantized EmbeddingBag of Section III-C: a table T of
 * 8-bit (or 4-bit) codes with one (scale, bias) pair per row; one lookup pools the rows named by
 * an index set I,
 *     R = sum_{i in I} scale[i] * T[i, :] + bias[i] * e_d          (optionally times a
 *     per-sample weight: the "weighted sum" of Section VI-A-2),
 * and the check compares RSum = sum_j R[j] against
 *     CSum = sum_{i in I} scale[i] * C_T[i] + d * bias[i]          (Eq. 4),
 * where C_T[i] = sum_j T[i][j] are 32-bit integer row sums computed once per table
 * (Section V: the table does not change after training, so the row sums are not part
 * of the overhead).  A batch applies the check to every lookup.
 *
 * What is fixed here where the paper leaves it open:
 *   - R is accumulated in binary32: per column one fused multiply-add per pooled row,
 *     in index order; the biases of a lookup are summed apart, in index order, and
 *     added to every column at the end.  With weights, scale and bias are first
 *     multiplied by the weight in binary32.
 *   - RSum and CSum are accumulated in binary64 (RSum over the binary32 values of R; CSum one
 *     term scale * C_T + d * bias per pooled row, each term rounded once; the order in which
 *     the terms are added is index order in one kernel and a tree in the other, a difference
 *     of at most n * 2^-53 * sum |term|).
 *   - err <=> not (|RSum - CSum| <= rel_bound * max(|RSum|, |CSum|)), or the difference is
 *     not finite.  The paper's choice is rel_bound = 1e-5 (Section V, round-off bound).
 *   - the row sums travel inside the table: a row is one record
 *     [d codes][scale f32][bias f32][C_T i32][4 bytes unused], d + 16 bytes for 8-bit codes, so
 *     the check reads no memory the lookup does not already touch.
 *
 * Conventions are those of abft_gemm.h: device pointers unless a comment says "host",
 * `stream` a hipStream_t passed as void*, calls enqueue and return, error codes and
 * abft_last_error() shared.  A DETECTED SOFT ERROR IS NOT AN ERROR RETURN: it is data
 * (bag_flags).
 */
#ifndef ABFT_EB_H
#define ABFT_EB_H

#include <stddef.h>
#include <stdint.h>

#include "abft_gemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* flags of abft_eb_u8_checked */
#define ABFT_EB_CHECK 0u          /* default: Algorithm 2 for every lookup */
#define ABFT_EB_NOCHECK 1u        /* same kernels with RSum, CSum and the comparison compiled out */
#define ABFT_EB_VARIANT_MASK 0xF00u /* 0 = choose by batch size */
#define ABFT_EB_VARIANT_BATCH 0x100u  /* a few lanes per lookup, rows straight into registers: large batches */
#define ABFT_EB_VARIANT_GROUP 0x200u  /* one workgroup per lookup, rows staged in LDS: small batches */

/* flags of abft_eb_pack_rowsum */
#define ABFT_EB_PACK_COMPACT 0u       /* default: records of d + 16 bytes back to back */
#define ABFT_EB_PACK_LINE_ALIGNED 1u  /* records of up to 128 bytes get a power-of-two stride (32, 64 or
                                         128 bytes), so that no record straddles a 128-byte memory
                                         line: fewer bytes fetched per lookup, a larger table */
#define ABFT_EB_PACK_INT4 2u          /* T holds 4-bit codes, two per byte, the even column in the low
                                         half (Section V, overhead analysis: p = 4 or 8 bits) */

/* bits of bag_flags[b] */
#define ABFT_EB_ERR 1          /* Algorithm 2's err: RSum and CSum differ by more than the bound */
#define ABFT_EB_BAD_INDEX 2    /* an index of the lookup lies outside the table; it was not pooled */

/* Opaque table: the fused row records described above.  The library owns its device memory; the table
 * belongs to the device that was current when it was built (a lookup with another device current
 * returns ABFT_EINVAL). */
typedef struct abft_eb_table abft_eb_table;

/* Section V, "pre-computed row sums of T": build the table once.
 *   T      the codes, rows x (d * bits / 8) bytes row-major with ldt (bytes) at least that
 *   scale, bias   float32 [rows]
 *   d      columns; a row of codes must be 16, 32, 64, 128, 256 or 512 bytes
 *          (d = 16 .. 512 for 8-bit codes, 32 .. 1024 for 4-bit codes, powers of two)
 *   out    host pointer receiving the handle
 *   flags  ABFT_EB_PACK_COMPACT, or ABFT_EB_PACK_LINE_ALIGNED and ABFT_EB_PACK_INT4 in any combination
 * Allocates rows * stride bytes with hipMalloc (stride = code bytes + 16 unless line-aligned); the packing
 * kernel is enqueued on `stream` and the inputs must stay valid until it has run. */
int abft_eb_pack_rowsum(const uint8_t* T, int64_t ldt, const float* scale, const float* bias, int64_t rows, int d,
                        unsigned flags, void* stream, abft_eb_table** out);

/* rows, d, the record stride in bytes and the code width in bits (host out-pointers, any may be NULL). */
int abft_eb_table_dims(const abft_eb_table* Tp, int64_t* rows, int* d, int* record_bytes, int* bits);

/* Copy C_T (int32 [rows]; Section V) out of the records. */
int abft_eb_table_get_rowsums(const abft_eb_table* Tp, int32_t* C_T, void* stream);

/* Fault-injection hook (Section VI-B-2: a random bit of a random element is flipped): inverts
 * bit `bit` (0..7, or 0..3 for 4-bit codes) of code T[row][col] inside the table and leaves C_T stale.  Calling it twice
 * with the same arguments restores the table. */
int abft_eb_table_flip_bit(abft_eb_table* Tp, int64_t row, int col, int bit, void* stream);

/* Host call.  Frees the handle; the caller has synchronised every stream that used it. */
void abft_eb_table_destroy(abft_eb_table* Tp);

/* Algorithm 2 for a batch of lookups.
 *   indices    int64 [n_indices]; offsets int64 [n_bags + 1], non-decreasing: lookup b pools
 *              indices[offsets[b] .. offsets[b+1]).  Offsets are clamped to [0, n_indices].
 *   weights    float32 [n_indices] per-sample weights, or NULL for the regular sum
 *   R          float32 n_bags x d row-major, ldr >= d, ldr a multiple of 4 and R 16-byte aligned
 *   bag_flags  int32 [n_bags]: ABFT_EB_ERR | ABFT_EB_BAD_INDEX (0 = clean).  With ABFT_EB_NOCHECK
 *              only ABFT_EB_BAD_INDEX is reported, and bag_flags may be NULL.
 *   rsum, csum float64 [n_bags] or NULL: the two sides of Eq. 4 as compared (diagnostics)
 *   rel_bound  the relative round-off bound of Algorithm 2 (the paper uses 1e-5)
 * An empty lookup gives a zero row and no error; n_bags == 0 is a valid call that does nothing.
 * No workspace, no host synchronisation. */
int abft_eb_u8_checked(const abft_eb_table* Tp, const int64_t* indices, int64_t n_indices, const int64_t* offsets,
                       int64_t n_bags, const float* weights, float* R, int64_t ldr, int32_t* bag_flags,
                       double* rsum, double* csum, double rel_bound, unsigned flags, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ABFT_EB_H */
