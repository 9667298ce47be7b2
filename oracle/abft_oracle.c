/*
 * CPU oracle for the ABFT-checked low-precision GEMM of arXiv 2103.00130
 * (Section IV, Algorithm 1; quantized product of Section III-A, Eq. 1).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * obviously-correct statement of what the method computes.  Only the tests,
 * the smoke check and the cpu_baseline leg of the benchmark may call it.  It
 * shares no code with the HIP path and knows nothing about tiles, packing
 * layouts, limbs or MFMA.
 *
 * Reading of the paper used throughout (the build's contract fixes the modulus):
 *   - the checksum column of B is kept as an exact int32 (Section IV: S_B[i] =
 *     sum_j B[i][j]) instead of being reduced mod 127 (Section IV-A-2), and the
 *     row check of Eq. 2b is an equality of two's-complement int32 values, i.e.
 *     an equality mod 2^32;
 *   - every sum below is taken in uint32_t so that wrap-around is defined C
 *     behaviour; a result is reinterpreted as int32 only when it is stored.
 * A second set of entry points (suffix _mod127) follows Algorithm 1 to the
 * letter: int8 checksum column reduced mod 127, comparison mod 127.
 *
 * Loops: i-k-j triple loop, OpenMP over rows only.  No blocking, no intrinsics.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Section IV, definition of the encoded column: S_B[k] = sum_j B[k][j]
 * (Algorithm 1, the loop that fills rowSum[], without the modulo step).
 * |S_B[k]| <= 128*N, exact in int32 for N < 2^24. */
void oracle_b_checksum(const int8_t* B, int64_t ldb, int K, int N, int32_t* S_B) {
    for (int k = 0; k < K; ++k) {
        uint32_t s = 0;
        for (int j = 0; j < N; ++j) s += (uint32_t)(int32_t)B[(int64_t)k * ldb + j];
        S_B[k] = (int32_t)s;
    }
}

/* Eq. 1, the rank-1 term e_k^T B_I: colsum[j] = sum_k B[k][j]. */
void oracle_b_colsum(const int8_t* B, int64_t ldb, int K, int N, int32_t* colsum) {
    for (int j = 0; j < N; ++j) {
        uint32_t s = 0;
        for (int k = 0; k < K; ++k) s += (uint32_t)(int32_t)B[(int64_t)k * ldb + j];
        colsum[j] = (int32_t)s;
    }
}

/* Section III-B: C_temp = A_I * B_I, A unsigned 8-bit, B signed 8-bit, 32-bit
 * accumulation (Algorithm 1, the product line, data columns only). */
void oracle_gemm_u8s8s32(const uint8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                         int M, int N, int K, int32_t* C, int64_t ldc) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        uint32_t* c = (uint32_t*)(C + (int64_t)i * ldc);
        for (int j = 0; j < N; ++j) c[j] = 0;
        for (int k = 0; k < K; ++k) {
            const uint32_t a = A[(int64_t)i * lda + k];
            const int8_t* b = B + (int64_t)k * ldb;
            for (int j = 0; j < N; ++j) c[j] += a * (uint32_t)(int32_t)b[j];
        }
    }
}

/* The extra column of C_temp in Algorithm 1: chk[i] = sum_k A[i][k] * S_B[k],
 * computed on its own from A and the stored checksum, never from C. */
void oracle_row_checksum(const uint8_t* A, int64_t lda, const int32_t* S_B, int M, int K,
                         int32_t* chk) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        uint32_t s = 0;
        for (int k = 0; k < K; ++k) s += (uint32_t)A[(int64_t)i * lda + k] * (uint32_t)S_B[k];
        chk[i] = (int32_t)s;
    }
}

/* Algorithm 1, tSum: rsum[i] = sum_{j<N} C[i][j]. */
void oracle_row_sums(const int32_t* C, int64_t ldc, int M, int N, int32_t* rsum) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        uint32_t s = 0;
        for (int j = 0; j < N; ++j) s += (uint32_t)C[(int64_t)i * ldc + j];
        rsum[i] = (int32_t)s;
    }
}

/* Algorithm 1, the comparison loop (Eq. 2b) with equality mod 2^32: flag[i] = 1
 * where the row sum and the checksum entry differ; returns errCount. */
int oracle_compare(const int32_t* rsum, const int32_t* chk, int M, int32_t* flags) {
    int count = 0;
    for (int i = 0; i < M; ++i) {
        flags[i] = (rsum[i] != chk[i]) ? 1 : 0;
        count += flags[i];
    }
    return count;
}

/* Requantization (Section III-B; Eq. 1 with beta_B = 0 and beta_A = -alpha_A*zA):
 *   t = C[i][j] - zA*colsum[j] (+ bias[j])      wrap-around int32
 *   y = clamp(round_half_even(t * mult) + zC, 0, 255)
 * mult is per tensor (per_channel = 0, mult[0]) or per output column.  The
 * checksum column never reaches this step (Section IV-A-3).  Arithmetic in
 * double: the exact product of an int32 and a float fits a double. */
void oracle_requantize_f64(const int32_t* C, int64_t ldc, int M, int N, const int32_t* colsum,
                           int32_t zA, int32_t zC, const float* mult, int per_channel,
                           const int32_t* bias, uint8_t* Cq, int64_t ldcq) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        for (int j = 0; j < N; ++j) {
            uint32_t t = (uint32_t)C[(int64_t)i * ldc + j] - (uint32_t)zA * (uint32_t)colsum[j];
            if (bias) t += (uint32_t)bias[j];
            const double m = (double)mult[per_channel ? j : 0];
            double y = nearbyint((double)(int32_t)t * m) + (double)zC;
            if (y < 0.0) y = 0.0;
            if (y > 255.0) y = 255.0;
            Cq[(int64_t)i * ldcq + j] = (uint8_t)y;
        }
    }
}

/* The same definition with every floating-point step in binary32 (int32 ->
 * float by round-to-nearest-even, one float multiply, rintf).  The rounding to
 * an 8-bit code is a decision taken in floating point, so the comparison with a
 * float32 kernel is made in the kernel's precision; the double version above
 * bounds how far that can drift (one code). */
void oracle_requantize_f32(const int32_t* C, int64_t ldc, int M, int N, const int32_t* colsum,
                           int32_t zA, int32_t zC, const float* mult, int per_channel,
                           const int32_t* bias, uint8_t* Cq, int64_t ldcq) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        for (int j = 0; j < N; ++j) {
            uint32_t t = (uint32_t)C[(int64_t)i * ldc + j] - (uint32_t)zA * (uint32_t)colsum[j];
            if (bias) t += (uint32_t)bias[j];
            volatile float tf = (float)(int32_t)t;
            volatile float p = tf * mult[per_channel ? j : 0];
            float r = rintf(p);
            /* r is integral and |r| < 2^31 * max(mult); clamp in float first. */
            float y = r + (float)zC;
            if (!(y >= 0.0f)) y = 0.0f;
            if (y > 255.0f) y = 255.0f;
            Cq[(int64_t)i * ldcq + j] = (uint8_t)y;
        }
    }
}

/* ---- Algorithm 1 as printed: modulus 127, 8-bit checksum column ------------------ */

static int32_t floor_mod127(int64_t v) {
    int64_t r = v % 127;
    if (r < 0) r += 127;
    return (int32_t)r;
}

/* rowSum[k] = (sum_j B[k][j]) mod 127, kept in [0,126] so it fits the signed
 * 8-bit container of B (Section IV-A-2).  The paper does not say which
 * representative "%" picks for a negative sum; the non-negative one is taken. */
void oracle_b_checksum_mod127(const int8_t* B, int64_t ldb, int K, int N, int8_t* rowSum) {
    for (int k = 0; k < K; ++k) {
        int64_t s = 0;
        for (int j = 0; j < N; ++j) s += B[(int64_t)k * ldb + j];
        rowSum[k] = (int8_t)floor_mod127(s);
    }
}

/* C_temp[i][n] of Algorithm 1 for the 8-bit column: sum_k A[i][k]*rowSum[k] in
 * 32-bit accumulation, like every other column of the product. */
void oracle_row_checksum_mod127(const uint8_t* A, int64_t lda, const int8_t* rowSum, int M, int K,
                                int32_t* chk) {
    for (int i = 0; i < M; ++i) {
        uint32_t s = 0;
        for (int k = 0; k < K; ++k)
            s += (uint32_t)A[(int64_t)i * lda + k] * (uint32_t)(int32_t)rowSum[k];
        chk[i] = (int32_t)s;
    }
}

/* The comparison of Algorithm 1: tSum % 127 != C_temp[i][n] % 127.  tSum is
 * summed without overflow (int64): 2^32 is not a multiple of 127, so a wrapped
 * 32-bit sum would break the congruence.  Both sides use the non-negative
 * representative, which is the reading under which a clean run never flags. */
int oracle_compare_mod127(const int32_t* C, int64_t ldc, int M, int N, const int32_t* chk,
                          int32_t* flags) {
    int count = 0;
    for (int i = 0; i < M; ++i) {
        int64_t t = 0;
        for (int j = 0; j < N; ++j) t += C[(int64_t)i * ldc + j];
        flags[i] = (floor_mod127(t) != floor_mod127(chk[i])) ? 1 : 0;
        count += flags[i];
    }
    return count;
}

/* ---- fault-injection campaigns (Section VI-B): each run recomputes, by the --------
 * ---- definitions above, exactly what the flipped element feeds ------------------- */

/* Bit flip in the 32-bit intermediate matrix: element (r,c) of a clean C has
 * bit `b` inverted before the row sums are taken.  For each injection the row
 * is copied, flipped, summed and compared with chk[r]; all other rows are
 * untouched.  out_flag[t] = verdict of row r; out_value[t] = the flipped element. */
void oracle_campaign_c_flips(const int32_t* C, int64_t ldc, int N, const int32_t* chk,
                             int n_inj, const int32_t* rows, const int32_t* cols,
                             const int32_t* bits, int32_t* out_flag, int32_t* out_value) {
#pragma omp parallel
    {
        uint32_t* row = (uint32_t*)malloc((size_t)N * sizeof(uint32_t));
#pragma omp for schedule(static)
        for (int t = 0; t < n_inj; ++t) {
            memcpy(row, C + (int64_t)rows[t] * ldc, (size_t)N * sizeof(uint32_t));
            row[cols[t]] ^= (uint32_t)1u << bits[t];
            uint32_t s = 0;
            for (int j = 0; j < N; ++j) s += row[j];
            out_flag[t] = ((int32_t)s != chk[rows[t]]) ? 1 : 0;
            out_value[t] = (int32_t)row[cols[t]];
        }
        free(row);
    }
}

/* Bit flip in B after its checksum was taken: B[k][j] ^= 1<<b, S_B stale.  Only
 * column j of C depends on B[k][j]; that column is recomputed from the flipped B
 * for every row, the row sums are re-taken over the whole row and compared with
 * the (unchanged) chk.  out_flags is [n_inj][M]; out_col is [n_inj][M], the
 * recomputed column.  C_clean is the product of the unflipped operands. */
void oracle_campaign_b_flips(const uint8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                             const int32_t* C_clean, int64_t ldc, int M, int N, int K,
                             const int32_t* chk, int n_inj, const int32_t* ks, const int32_t* js,
                             const int32_t* bits, int32_t* out_flags, int32_t* out_col) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n_inj; ++t) {
        const int kf = ks[t], jf = js[t];
        const int8_t flipped = (int8_t)((uint8_t)B[(int64_t)kf * ldb + jf] ^ (uint8_t)(1u << bits[t]));
        for (int i = 0; i < M; ++i) {
            uint32_t c = 0;
            for (int k = 0; k < K; ++k) {
                const int8_t b = (k == kf) ? flipped : B[(int64_t)k * ldb + jf];
                c += (uint32_t)A[(int64_t)i * lda + k] * (uint32_t)(int32_t)b;
            }
            uint32_t s = 0;
            for (int j = 0; j < N; ++j)
                s += (j == jf) ? c : (uint32_t)C_clean[(int64_t)i * ldc + j];
            out_col[(int64_t)t * M + i] = (int32_t)c;
            out_flags[(int64_t)t * M + i] = ((int32_t)s != chk[i]) ? 1 : 0;
        }
    }
}

/* The same B-fault campaign under Algorithm 1 as printed: chk is the product with the
 * 8-bit column rowSum = S_B mod 127 (stale after the flip), the row sums are taken without
 * overflow and the comparison is modulo 127.  out_flags and out_col are [n_inj][M]. */
void oracle_campaign_b_flips_mod127(const uint8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                                    const int32_t* C_clean, int64_t ldc, int M, int N, int K,
                                    const int32_t* chk127, int n_inj, const int32_t* ks,
                                    const int32_t* js, const int32_t* bits, int32_t* out_flags,
                                    int32_t* out_col) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n_inj; ++t) {
        const int kf = ks[t], jf = js[t];
        const int8_t flipped = (int8_t)((uint8_t)B[(int64_t)kf * ldb + jf] ^ (uint8_t)(1u << bits[t]));
        for (int i = 0; i < M; ++i) {
            uint32_t c = 0;
            for (int k = 0; k < K; ++k) {
                const int8_t b = (k == kf) ? flipped : B[(int64_t)k * ldb + jf];
                c += (uint32_t)A[(int64_t)i * lda + k] * (uint32_t)(int32_t)b;
            }
            int64_t s = 0;
            for (int j = 0; j < N; ++j)
                s += (j == jf) ? (int32_t)c : C_clean[(int64_t)i * ldc + j];
            out_col[(int64_t)t * M + i] = (int32_t)c;
            out_flags[(int64_t)t * M + i] = (floor_mod127(s) != floor_mod127(chk127[i])) ? 1 : 0;
        }
    }
}

/* The second fault model of Section IV-C (an element takes an arbitrary wrong value) and
 * multi-bit upsets, in the 32-bit intermediate: element (r,c) of a clean C is XOR-ed with
 * `mask` (mask = old ^ new for a replacement) before the row sums are taken.  Same procedure
 * as for single bits: the row is copied, changed, summed and compared with chk[r]. */
void oracle_campaign_c_masks(const int32_t* C, int64_t ldc, int N, const int32_t* chk,
                             int n_inj, const int32_t* rows, const int32_t* cols,
                             const uint32_t* masks, int32_t* out_flag, int32_t* out_value) {
#pragma omp parallel
    {
        uint32_t* row = (uint32_t*)malloc((size_t)N * sizeof(uint32_t));
#pragma omp for schedule(static)
        for (int t = 0; t < n_inj; ++t) {
            memcpy(row, C + (int64_t)rows[t] * ldc, (size_t)N * sizeof(uint32_t));
            row[cols[t]] ^= masks[t];
            uint32_t s = 0;
            for (int j = 0; j < N; ++j) s += row[j];
            out_flag[t] = ((int32_t)s != chk[rows[t]]) ? 1 : 0;
            out_value[t] = (int32_t)row[cols[t]];
        }
        free(row);
    }
}

/* The same two models in B after its checksum was taken: B[k][j] takes the value
 * new_vals[t] (any int8), S_B stale.  Column j of C is recomputed from the changed B for
 * every row, the row sums are re-taken over the whole row and compared with the
 * (unchanged) chk.  out_flags and out_col are [n_inj][M]. */
void oracle_campaign_b_values(const uint8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                              const int32_t* C_clean, int64_t ldc, int M, int N, int K,
                              const int32_t* chk, int n_inj, const int32_t* ks, const int32_t* js,
                              const int32_t* new_vals, int32_t* out_flags, int32_t* out_col) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n_inj; ++t) {
        const int kf = ks[t], jf = js[t];
        const int8_t changed = (int8_t)new_vals[t];
        for (int i = 0; i < M; ++i) {
            uint32_t c = 0;
            for (int k = 0; k < K; ++k) {
                const int8_t b = (k == kf) ? changed : B[(int64_t)k * ldb + jf];
                c += (uint32_t)A[(int64_t)i * lda + k] * (uint32_t)(int32_t)b;
            }
            uint32_t s = 0;
            for (int j = 0; j < N; ++j)
                s += (j == jf) ? c : (uint32_t)C_clean[(int64_t)i * ldc + j];
            out_col[(int64_t)t * M + i] = (int32_t)c;
            out_flags[(int64_t)t * M + i] = ((int32_t)s != chk[i]) ? 1 : 0;
        }
    }
}

/* Bit flip in A before the product: A[i][k] ^= 1<<b.  Row i of C and chk[i] are
 * both recomputed from the flipped A (A is not encoded, Section IV-C-3), the
 * row is summed and compared.  out_flag[t] = verdict of row i; out_row, when
 * not NULL, is [n_inj][N] and receives the recomputed row of C. */
void oracle_campaign_a_flips(const uint8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                             const int32_t* S_B, int N, int K, int n_inj, const int32_t* is,
                             const int32_t* ks, const int32_t* bits, int32_t* out_flag,
                             int32_t* out_row) {
#pragma omp parallel
    {
        uint8_t* a = (uint8_t*)malloc((size_t)K);
        uint32_t* local = (uint32_t*)malloc((size_t)N * sizeof(uint32_t));
#pragma omp for schedule(dynamic, 4)
        for (int t = 0; t < n_inj; ++t) {
            memcpy(a, A + (int64_t)is[t] * lda, (size_t)K);
            a[ks[t]] ^= (uint8_t)(1u << bits[t]);
            uint32_t* c = out_row ? (uint32_t*)(out_row + (int64_t)t * N) : local;
            for (int j = 0; j < N; ++j) c[j] = 0;
            uint32_t chk = 0;
            for (int k = 0; k < K; ++k) {
                const uint32_t av = a[k];
                const int8_t* b = B + (int64_t)k * ldb;
                for (int j = 0; j < N; ++j) c[j] += av * (uint32_t)(int32_t)b[j];
                chk += av * (uint32_t)S_B[k];
            }
            uint32_t s = 0;
            for (int j = 0; j < N; ++j) s += c[j];
            out_flag[t] = (s != chk) ? 1 : 0;
        }
        free(local);
        free(a);
    }
}

/* ---- Locating and correcting a single faulty element (Section IV, Eq. 2a and the two ----
 * ---- correction formulas that follow the pair of checks)                              ----
 * The full scheme encodes A as well: S_A[k] = sum_i A[i][k] (the appended row of A'), whose
 * product with B is the extra row of C', C'[m][j] = (S_A B)[j].  Eq. 2a: every column of a
 * correct C sums to that entry.  All sums modulo 2^32, like the row check. */

/* S_A[k] = sum_i A[i][k] (Section IV, definition of the row appended to A). */
void oracle_a_colsum(const uint8_t* A, int64_t lda, int M, int K, int32_t* S_A) {
    for (int k = 0; k < K; ++k) {
        uint32_t s = 0;
        for (int i = 0; i < M; ++i) s += (uint32_t)A[(int64_t)i * lda + k];
        S_A[k] = (int32_t)s;
    }
}

/* C'[m][j] = sum_k S_A[k] * B[k][j]: the checksum row, computed on its own (not from C). */
void oracle_col_checksum(const int32_t* S_A, const int8_t* B, int64_t ldb, int K, int N, int32_t* col_chk) {
    for (int j = 0; j < N; ++j) {
        uint32_t s = 0;
        for (int k = 0; k < K; ++k) s += (uint32_t)S_A[k] * (uint32_t)(int32_t)B[(int64_t)k * ldb + j];
        col_chk[j] = (int32_t)s;
    }
}

/* Right-hand side of Eq. 2a: csum[j] = sum_i C[i][j]. */
void oracle_col_sums(const int32_t* C, int64_t ldc, int M, int N, int32_t* csum) {
    for (int j = 0; j < N; ++j) {
        uint32_t s = 0;
        for (int i = 0; i < M; ++i) s += (uint32_t)C[(int64_t)i * ldc + j];
        csum[j] = (int32_t)s;
    }
}

/* The decision and the repair (text after Eq. 2b): with exactly one row i violating Eq. 2b and
 * exactly one column j violating Eq. 2a the element C[i][j] is the faulty one, and
 *     correct C[i][j] = C'[m][j] - sum_{p != i} C[p][j]      (first formula)
 *                     = C'[i][n] - sum_{p != j} C[i][p]      (second formula).
 * C is repaired in place with the first formula; the second is evaluated too and the pair must agree,
 * otherwise nothing is written (a pattern that is not one faulty element of C).
 * row_flags: the verdicts of Eq. 2b as the checked product returned them; row_chk[i] = (A S_B)[i].
 * out[0] = status: 0 nothing violated, 1 located and corrected, 2 violations that do not single out
 * one element (C untouched); out[1], out[2] = row, column (status 1, else -1); out[3], out[4] = value
 * found there and value written; out[5], out[6] = number of violated rows and columns. */
void oracle_locate_correct(int32_t* C, int64_t ldc, int M, int N, const int32_t* row_flags, const int32_t* row_chk,
                           const int32_t* col_chk, int32_t* col_flags, int32_t* out) {
    int n_rows = 0, n_cols = 0, row = -1, col = -1;
    for (int i = 0; i < M; ++i)
        if (row_flags[i] != 0) { ++n_rows; row = i; }
    for (int j = 0; j < N; ++j) {
        uint32_t s = 0;
        for (int i = 0; i < M; ++i) s += (uint32_t)C[(int64_t)i * ldc + j];
        col_flags[j] = (int32_t)s != col_chk[j];
        if (col_flags[j]) { ++n_cols; col = j; }
    }
    out[0] = (n_rows == 0 && n_cols == 0) ? 0 : 2;
    out[1] = out[2] = -1;
    out[3] = out[4] = 0;
    out[5] = n_rows;
    out[6] = n_cols;
    if (n_rows != 1 || n_cols != 1) return;
    uint32_t others_in_col = 0, others_in_row = 0;
    for (int p = 0; p < M; ++p)
        if (p != row) others_in_col += (uint32_t)C[(int64_t)p * ldc + col];
    for (int p = 0; p < N; ++p)
        if (p != col) others_in_row += (uint32_t)C[(int64_t)row * ldc + p];
    const int32_t by_column = (int32_t)((uint32_t)col_chk[col] - others_in_col);
    const int32_t by_row = (int32_t)((uint32_t)row_chk[row] - others_in_row);
    if (by_column != by_row) return;
    out[0] = 1;
    out[1] = row;
    out[2] = col;
    out[3] = C[(int64_t)row * ldc + col];
    out[4] = by_column;
    C[(int64_t)row * ldc + col] = by_column;
}
