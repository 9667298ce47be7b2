/*
 * CPU oracle for the ABFT-checked low-precision EmbeddingBag of arXiv 2103.00130
 * (operator: Section III-C; check: Section V, Eq. 4 and Algorithm 2).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Plain loops that state what the
 * method computes.  Only the tests, the smoke check and the cpu_baseline leg of the
 * benchmark may call it.  It shares no code with the HIP path and knows nothing
 * about fused row records, lanes or wavefronts.
 *
 * Tables hold 8-bit codes (one per byte) or 4-bit codes (Section V, overhead analysis: p = 4 or 8
 * bits; two codes per byte, the even column in the low half): `bits` says which, and a row of
 * the table is d * bits / 8 bytes.
 *
 * Notation of the paper: T the table of 8-bit codes, d its row length, alpha[i] and
 * beta[i] the scale and bias of row i, I the index set of one lookup ("bag"), R the
 * pooled row, C_T[i] = sum_j T[i][j] the precomputed 32-bit integer row sums.
 * A batch is n_bags index sets in the offsets form: bag b pools
 * indices[offsets[b] .. offsets[b+1]).  The weighted sum multiplies every pooled
 * row by a per-sample weight w (Section VI-A-2 measures both).
 *
 * Readings where the paper is silent:
 *  - R is evaluated in two precisions.  _f64 is the definition in double.  _f32 is
 *    the paper's precision (float): per column, one fused multiply-add
 *    acc = alpha*code + acc per pooled row, in index order; the biases of the bag
 *    are summed separately, in index order, and added to every column at the end
 *    (R = sum alpha*eb + (sum beta) e_d, the same sum regrouped).  With weights,
 *    alpha and beta are first multiplied by w in float.
 *  - RSum and CSum of Algorithm 2 are accumulated in double (RSum over the float
 *    values of R); the integer row sums enter CSum unscaled, as Section V states.
 *    CSum adds one term per pooled row, the parenthesised (alpha * C_T + d * beta)
 *    of Algorithm 2's third step formed first (both products are exact in double,
 *    so the term is their sum rounded once).
 *  - "relative bound": err <=> not (|RSum - CSum| <= bound * max(|RSum|, |CSum|)), or
 *    |RSum - CSum| not finite, so that a NaN or an infinity on either side reports an error.
 *  - an index outside [0, rows) is not pooled and sets bit 1 (value 2) of the bag's
 *    flag; bit 0 is Algorithm 2's err.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline int code_at(const uint8_t* T, int64_t i, int j, int d, int bits) {
    if (bits == 8) return T[i * d + j];
    const uint8_t b = T[i * (d / 2) + (j >> 1)];
    return (j & 1) ? (b >> 4) : (b & 15);
}

/* Section V: the column vector C_T of row sums of the table, 32-bit integers. */
void eb_oracle_rowsums(const uint8_t* T, int64_t rows, int d, int bits, int32_t* C_T) {
    for (int64_t i = 0; i < rows; ++i) {
        int32_t s = 0;
        for (int j = 0; j < d; ++j) s += code_at(T, i, j, d, bits);
        C_T[i] = s;
    }
}

/* Section III-C: R = sum_{i in I} alpha_i eb_i + beta_i e_d (times w_i when weighted), in double. */
void eb_oracle_forward_f64(const uint8_t* T, int64_t rows, int d, int bits, const float* alpha, const float* beta,
                           const int64_t* indices, const int64_t* offsets, int64_t n_bags, const float* w, double* R) {
    for (int64_t b = 0; b < n_bags; ++b) {
        for (int j = 0; j < d; ++j) R[b * d + j] = 0.0;
        for (int64_t p = offsets[b]; p < offsets[b + 1]; ++p) {
            const int64_t i = indices[p];
            if (i < 0 || i >= rows) continue;
            const double wi = w ? (double)w[p] : 1.0;
            for (int j = 0; j < d; ++j)
                R[b * d + j] += wi * ((double)alpha[i] * (double)code_at(T, i, j, d, bits) + (double)beta[i]);
        }
    }
}

/* The same in float, in the order stated in the header.  This is a regrouping of the definition
 * (one fma per column and row, biases summed apart): tests use it to check that an implementation
 * reproduces that documented order bit for bit.  The parity reference is _f64 above. */
void eb_oracle_forward_f32(const uint8_t* T, int64_t rows, int d, int bits, const float* alpha, const float* beta,
                           const int64_t* indices, const int64_t* offsets, int64_t n_bags, const float* w, float* R) {
    for (int64_t b = 0; b < n_bags; ++b) {
        for (int j = 0; j < d; ++j) R[b * d + j] = 0.0f;
        float beta_sum = 0.0f;
        for (int64_t p = offsets[b]; p < offsets[b + 1]; ++p) {
            const int64_t i = indices[p];
            if (i < 0 || i >= rows) continue;
            const float a = w ? w[p] * alpha[i] : alpha[i];
            const float c = w ? w[p] * beta[i] : beta[i];
            for (int j = 0; j < d; ++j) R[b * d + j] = fmaf(a, (float)code_at(T, i, j, d, bits), R[b * d + j]);
            beta_sum = beta_sum + c;
        }
        for (int j = 0; j < d; ++j) R[b * d + j] = R[b * d + j] + beta_sum;
    }
}

/* Algorithm 2, the steps after the lookup: RSum, CSum (Eq. 4), comparison against the
 * round-off bound.  R is the float result of the lookup (ldr floats per bag). */
void eb_oracle_check(const float* R, int64_t ldr, int64_t rows, int d, const float* alpha, const float* beta,
                     const int32_t* C_T, const int64_t* indices, const int64_t* offsets, int64_t n_bags,
                     const float* w, double bound, int32_t* flags, double* rsum_out, double* csum_out) {
    for (int64_t b = 0; b < n_bags; ++b) {
        double rsum = 0.0, csum = 0.0;
        int32_t flag = 0;
        for (int j = 0; j < d; ++j) rsum += (double)R[b * ldr + j];
        for (int64_t p = offsets[b]; p < offsets[b + 1]; ++p) {
            const int64_t i = indices[p];
            if (i < 0 || i >= rows) {
                flag |= 2;
                continue;
            }
            const float a = w ? w[p] * alpha[i] : alpha[i];
            const float c = w ? w[p] * beta[i] : beta[i];
            csum += (double)a * (double)C_T[i] + (double)d * (double)c;
        }
        const double diff = fabs(rsum - csum);
        if (!(diff <= bound * fmax(fabs(rsum), fabs(csum))) || !(diff < INFINITY)) flag |= 1;
        flags[b] = flag;
        if (rsum_out) rsum_out[b] = rsum;
        if (csum_out) csum_out[b] = csum;
    }
}

/* Section VI-B-2: one bit of one table element is flipped after C_T was computed, the batch is
 * looked up and checked (in float), the element is restored.  f_bit counts inside the element
 * (0..bits-1).  flags_out[n][n_bags]. */
void eb_oracle_campaign_table_flips(uint8_t* T, int64_t rows, int d, int bits, const float* alpha, const float* beta,
                                    const int32_t* C_T, const int64_t* indices, const int64_t* offsets, int64_t n_bags,
                                    const float* w, double bound, const int64_t* f_row, const int32_t* f_col,
                                    const int32_t* f_bit, int64_t n, int32_t* flags_out) {
    float* R = (float*)malloc(sizeof(float) * (size_t)n_bags * (size_t)d);
    for (int64_t t = 0; t < n; ++t) {
        /* the element's bit inside its byte: a 4-bit code of an odd column sits in the high half */
        uint8_t* e = bits == 8 ? &T[f_row[t] * d + f_col[t]] : &T[f_row[t] * (d / 2) + (f_col[t] >> 1)];
        const uint8_t mask = (uint8_t)(1u << (f_bit[t] + (bits == 4 && (f_col[t] & 1) ? 4 : 0)));
        *e ^= mask;
        eb_oracle_forward_f32(T, rows, d, bits, alpha, beta, indices, offsets, n_bags, w, R);
        eb_oracle_check(R, d, rows, d, alpha, beta, C_T, indices, offsets, n_bags, w, bound, flags_out + t * n_bags, 0, 0);
        *e ^= mask;
    }
    free(R);
}
