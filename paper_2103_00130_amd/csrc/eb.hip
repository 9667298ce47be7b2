// ABFT-checked row-wise quantized EmbeddingBag (include/abft_eb.h): Algorithm 2 of
// arXiv 2103.00130 (Section V) on the operator of Section III-C.
//
// The work is a gather: every pooled row is read once from a table far larger than any
// cache, so the kernels are built around bytes in flight, not arithmetic.
//
//  * Codes are 8 bits wide, or 4 bits wide and packed two per byte (Section V: p = 4 or 8); the
//    kernels are templated on the width and differ only in how a code is cut out of its word.
//  * The table is kept as fused records [codes][scale][bias][C_T][unused]: the row sum that
//    Eq. 4 needs arrives in the same memory transaction as the scale and bias the lookup needs
//    anyway, so the check adds no memory traffic at all.
//  * Batch kernel (large batches): one lane per 16 code bytes of a row.  Every lane owns the columns
//    of its bytes and reads them per pooled row straight into registers, eight rows in flight per
//    lane; the chip is filled by lookups, and the lanes of a lookup walk its index list in order.
//  * Group kernel (small batches): one workgroup per lookup.  All threads fetch different 16-byte
//    pieces of the lookup's records into LDS (1024 or 2048 pieces in flight per workgroup), then
//    the threads, now owning columns, walk the staged rows in index order.
//  * Every load is unconditional (clamped position, row 0 in place of a bad index): a load under
//    `if (valid)` is followed by a wait, which would put the loads of a lookup one after the other.
//  Both accumulate every output column in the same order (index order, one fused multiply-add
//  per row, biases summed apart), so they give the same bits; RSum and CSum are taken in
//  binary64.  CSum adds one exactly rounded term per pooled row: in index order in the batch
//  kernel, lanes in parallel (a tree) in the group kernel - Eq. 4 fixes the terms, not their order.
#include <cmath>
#include <cstring>
#include <new>

#include "../../include/abft_eb.h"
#include "abft_internal.h"

struct abft_eb_table {
    uint8_t* rec;    // rows * stride bytes: [codes][scale f32][bias f32][C_T i32][unused]
    int64_t rows;
    int64_t stride;  // code bytes + 16, or the next power of two when the records are line-aligned
    int d;           // columns
    int bits;        // 8 or 4 bits per code
    int code_bytes;  // d * bits / 8
    int device;
};

namespace abft {
namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct EbParams {
    const uint8_t* tab;
    int64_t stride;  // bytes from one record to the next
    int64_t rows;
    const int64_t* indices;
    int64_t n_indices;
    const int64_t* offsets;
    int64_t n_bags;
    const float* weights;
    float* R;
    int64_t ldr;
    int32_t* flags;
    double* rsum;
    double* csum;
    double bound;
};

__device__ inline float as_f32(unsigned int u) { return __builtin_bit_cast(float, u); }

__device__ inline void bag_range(const EbParams& p, int64_t bag, int64_t* beg, int64_t* end) {
    int64_t b = p.offsets[bag], e = p.offsets[bag + 1];
    b = b < 0 ? 0 : (b > p.n_indices ? p.n_indices : b);
    e = e < b ? b : (e > p.n_indices ? p.n_indices : e);
    *beg = b;
    *end = e;
}

// Algorithm 2, the comparison: err unless |RSum - CSum| <= bound * max(|RSum|, |CSum|) and finite
__device__ inline int compare_sums(double rs, double cs, double bound) {
    const double diff = fabs(rs - cs);
    return (!(diff <= bound * fmax(fabs(rs), fabs(cs))) || !(diff < (double)INFINITY)) ? ABFT_EB_ERR : 0;
}

// Value that lane ^ M holds, without a trip through memory: DPP inside a row of 16 lanes, the swizzle
// crossbar for M = 4 and 8, the row and half swaps beyond (both give {own, partner} in an order that
// depends on the lane, hence the XOR).
template <int M>
__device__ inline unsigned int from_lane_xor(unsigned int v) {
    static_assert(M == 1 || M == 2 || M == 4 || M == 8 || M == 16 || M == 32, "one bit of the lane number");
    if constexpr (M == 1) return (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    else if constexpr (M == 2) return (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    else if constexpr (M == 4) return (unsigned int)__builtin_amdgcn_ds_swizzle((int)v, 0x101F);
    else if constexpr (M == 8) return (unsigned int)__builtin_amdgcn_ds_swizzle((int)v, 0x201F);
    else if constexpr (M == 16) {
        const auto sw = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        return sw[0] ^ sw[1] ^ v;
    } else {
        const auto sw = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return sw[0] ^ sw[1] ^ v;
    }
}

template <int M>
__device__ inline double from_lane_xor(double v) {
    const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
    const unsigned long long o = (unsigned long long)from_lane_xor<M>((unsigned int)b) |
                                 ((unsigned long long)from_lane_xor<M>((unsigned int)(b >> 32)) << 32);
    return __builtin_bit_cast(double, o);
}

// sum over the 64 lanes, the same value in every lane: a butterfly (lane pairs, then pairs of pairs, ...)
__device__ inline double wave_sum(double v) {
    v += from_lane_xor<1>(v);
    v += from_lane_xor<2>(v);
    v += from_lane_xor<4>(v);
    v += from_lane_xor<8>(v);
    v += from_lane_xor<16>(v);
    v += from_lane_xor<32>(v);
    return v;
}

// the columns held by 16 code bytes of one pooled row: acc[k] = a * code[k] + acc[k].
// 8-bit codes: 16 columns; 4-bit codes: 32 columns, the even column in the low half of its byte.
template <int BITS>
__device__ inline void fma_codes(float (&acc)[128 / BITS], float a, v4u q) {
    constexpr int PER_WORD = 32 / BITS;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int n = 0; n < PER_WORD; ++n)
            acc[PER_WORD * w + n] = __builtin_fmaf(a, (float)((q[w] >> (BITS * n)) & ((1u << BITS) - 1u)), acc[PER_WORD * w + n]);
}

// ---------------------------------------------------------------------------------------------
// Batch kernel: G lanes per lookup, one per 16 code bytes of a row.
template <int G, int BITS, bool kCheck, bool kWeighted, bool kTwoSets>
__global__ __launch_bounds__(256) void eb_batch_kernel(const EbParams p) {
    constexpr int CB = 16 * G;            // code bytes per row
    constexpr int CPP = 128 / BITS;       // columns per 16-byte piece
    constexpr int D = G * CPP, U = 8;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t bag = t / G;
    const int piece = (int)(t % G);
    if (bag >= p.n_bags) return;  // whole lane groups leave together (256 is a multiple of G)
    int64_t beg, end;
    bag_range(p, bag, &beg, &end);

    float acc[CPP];
#pragma unroll
    for (int k = 0; k < CPP; ++k) acc[k] = 0.0f;
    float beta_sum = 0.0f;
    double cs = 0.0;
    int flag = 0;
    const uint8_t* const base = p.tab + piece * 16;

    // Rows are handled in sets of U.  Every load is unconditional inside its set (clamped position,
    // row 0 in place of a bad index): the index loads of a set go out together, then its row loads,
    // and only then anything waits.
    // kTwoSets: two sets in flight - the row loads of a set go out while the set before it is being
    // pooled, and the indices of the set after it are already on their way - so that the latency of
    // the indices, the latency of the rows and the arithmetic overlap instead of adding up.  A launch
    // of a few wavefronts per SIMD has nothing else to hide them behind; with many wavefronts the
    // other wavefronts do that, and the registers of the second set cost more than it gains.
    // A row that is not pooled enters the sums with scale, bias and row sum 0, which leaves every
    // accumulator as it is, bit for bit.
    struct IdxSet {
        int64_t idx[U];
        float wv[U];
    };
    struct RowSet {
        float wv[U];
        v4u q[U], tl[U];
        bool ok[U];
    };
    auto load_indices = [&](IdxSet& r, int64_t pos) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t pp = pos + u < end ? pos + u : end - 1;
            r.idx[u] = p.indices[pp];
            if (kWeighted) r.wv[u] = p.weights[pp];
        }
    };
    auto load_rows = [&](RowSet& r, const IdxSet& ix, int64_t pos) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool in = pos + u < end;
            r.ok[u] = in && (uint64_t)ix.idx[u] < (uint64_t)p.rows;
            if (in && !r.ok[u]) flag |= ABFT_EB_BAD_INDEX;
            if (kWeighted) r.wv[u] = ix.wv[u];
            const uint8_t* rec = base + (r.ok[u] ? ix.idx[u] : 0) * p.stride;
            r.q[u] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(rec));
            r.tl[u] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(rec + (CB - piece * 16)));
        }
    };
    auto pool = [&](const RowSet& r) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float a = as_f32(r.tl[u][0]), c = as_f32(r.tl[u][1]);
            if (kWeighted) {
                a = r.wv[u] * a;
                c = r.wv[u] * c;
            }
            a = r.ok[u] ? a : 0.0f;
            c = r.ok[u] ? c : 0.0f;
            fma_codes<BITS>(acc, a, r.q[u]);
            beta_sum = beta_sum + c;
            if (kCheck) {
                // Eq. 4, the term of one pooled row: scale * C_T + d * bias, rounded once (both products
                // are exact in binary64), then added to the running sum
                cs = cs + fma((double)a, (double)(r.ok[u] ? (int32_t)r.tl[u][2] : 0), (double)D * (double)c);
            }
        }
    };
    if (!kTwoSets) {
        for (int64_t pos = beg; pos < end; pos += U) {
            IdxSet ia;
            RowSet ra;
            load_indices(ia, pos);
            load_rows(ra, ia, pos);
            pool(ra);
        }
    } else if (beg < end) {
        IdxSet ia, ib;
        RowSet ra, rb;
        load_indices(ia, beg);
        load_rows(ra, ia, beg);
        load_indices(ib, beg + U);
        for (int64_t pos = beg;; pos += 2 * U) {
            // here the rows of ra and the indices ib are in flight
            if (pos + U < end) {
                load_rows(rb, ib, pos + U);
                load_indices(ia, pos + 2 * U);
            }
            pool(ra);
            if (pos + U >= end) break;
            if (pos + 2 * U < end) {
                load_rows(ra, ia, pos + 2 * U);
                load_indices(ib, pos + 3 * U);
            }
            pool(rb);
            if (pos + 2 * U >= end) break;
        }
    }

    float* const out = p.R + bag * p.ldr + piece * CPP;
    double rs = 0.0;
#pragma unroll
    for (int w = 0; w < CPP / 4; ++w) {
        v4f v;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = acc[4 * w + k] + beta_sum;
            if (kCheck) rs += (double)v[k];
        }
        *reinterpret_cast<v4f*>(out + 4 * w) = v;
    }
    if (kCheck) {
        if constexpr (G > 1) rs += from_lane_xor<1>(rs);
        if constexpr (G > 2) rs += from_lane_xor<2>(rs);
        if constexpr (G > 4) rs += from_lane_xor<4>(rs);
        if constexpr (G > 8) rs += from_lane_xor<8>(rs);
        if constexpr (G > 16) rs += from_lane_xor<16>(rs);
        if (piece == 0) {
            p.flags[bag] = flag | compare_sums(rs, cs, p.bound);
            if (p.rsum) p.rsum[bag] = rs;
            if (p.csum) p.csum[bag] = cs;
        }
    } else if (p.flags && piece == 0) {
        p.flags[bag] = flag;
    }
}

// ---------------------------------------------------------------------------------------------
// Group kernel: one workgroup (four wavefronts) per lookup, rows staged through LDS.
//  1. fetch: every thread loads different 16-byte pieces of the chunk's records (1024 pieces in
//     flight per workgroup) and they are laid out in LDS record after record;
//  2. per-row scalars, rows in parallel: the weighted scale and bias of every staged row, and
//     the two exact binary64 products of its Eq. 4 term;
//  3. pooling, rows in index order: threads own columns and do one LDS read, one convert and one
//     fused multiply-add per row; meanwhile the last two wavefronts form the sums that do not
//     depend on the column (the biases, in index order like the columns; the terms of CSum, lanes
//     in parallel).
template <int G, int BITS, bool kCheck, bool kWeighted>
__global__ __launch_bounds__(256) void eb_group_kernel(const EbParams p) {
    constexpr int CB = 16 * G;                 // code bytes per row
    constexpr int D = CB * 8 / BITS, REC = CB + 16;   // REC: a record as staged in LDS (no padding there)
    constexpr int P = G + 1;                   // 16-byte pieces per record
    constexpr int NL = G >= 16 ? 8 : 4;        // load instructions per thread and chunk
    constexpr int PIECES = NL * 256;
    constexpr int ROWS = PIECES / P;           // whole records per chunk
    constexpr int NW = (ROWS + 255) / 256;     // rows per thread in the per-row pass
    constexpr int BPT = CB > 256 ? CB / 256 : 1;  // code bytes per thread in the pooling phase
    constexpr int CPL = BPT * 8 / BITS;           // columns per thread
    // (the per-row scalars replace the tail piece of their staged record: no LDS beyond the records,
    // so that eight workgroups - all the wavefront slots - fit a compute unit at every row width)
    __shared__ v4u s_rec[PIECES];
    __shared__ double s_rs[4], s_cs;
    __shared__ float s_beta;
    __shared__ int s_flag;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bag = blockIdx.x;
    int64_t beg, end;
    bag_range(p, bag, &beg, &end);

    float acc[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) acc[k] = 0.0f;
    float beta_sum = 0.0f;
    double cs = 0.0;
    const bool col_thread = tid * BPT < CB;
    // the chains that do not depend on the column run on wavefronts that own few or no columns
    const bool beta_wave = wave == 2, cs_wave = wave == 3;
    const uint8_t* const s_bytes = reinterpret_cast<const uint8_t*>(s_rec);
    // staged tail of row r after the per-row pass: [weighted scale f32][weighted bias f32][Eq. 4 term f64]
    auto row_scale = [&](int r) __attribute__((always_inline)) { return *reinterpret_cast<const float*>(s_bytes + r * REC + CB); };
    auto row_bias = [&](int r) __attribute__((always_inline)) { return *reinterpret_cast<const float*>(s_bytes + r * REC + CB + 4); };
    auto row_term = [&](int r) __attribute__((always_inline)) { return *reinterpret_cast<const double*>(s_bytes + r * REC + CB + 8); };
    if (tid == 0) s_flag = 0;

    for (int64_t pos = beg; pos < end; pos += ROWS) {
        const int n = (int)(end - pos < ROWS ? end - pos : ROWS);
        // fetch: piece g = l*256 + tid of the chunk is piece g % P of row g / P.  All loads are
        // unconditional (clamped row, row 0 in place of a bad index) so that they all go out together.
        int64_t idx[NL];
#pragma unroll
        for (int l = 0; l < NL; ++l) {
            const int r = (l * 256 + tid) / P;
            idx[l] = p.indices[pos + (r < n ? r : n - 1)];
        }
        float wreg[NW];
        if (kWeighted)
#pragma unroll
            for (int k = 0; k < NW; ++k) wreg[k] = p.weights[pos + (tid + 256 * k < n ? tid + 256 * k : n - 1)];
        v4u v[NL];
#pragma unroll
        for (int l = 0; l < NL; ++l) {
            const int g = l * 256 + tid, r = g / P, pc = g - r * P;
            const bool ok = (uint64_t)idx[l] < (uint64_t)p.rows;
            v[l] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p.tab + (ok ? idx[l] : 0) * p.stride + pc * 16));
            // the last word of a record's tail is unused in memory; staged, it marks a row that is not pooled
            if (pc == G) v[l][3] = ok ? 0u : 1u;
        }
        __syncthreads();  // the previous chunk has been pooled
#pragma unroll
        for (int l = 0; l < NL; ++l) s_rec[l * 256 + tid] = v[l];
        __syncthreads();
        // per-row scalars.  A row that is not pooled gets scale, bias and row sum 0, which leaves every
        // accumulator as it is, bit for bit.
        int bad_any = 0;
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            const int r = tid + 256 * k;
            if (r < n) {
                const v4u tl = s_rec[r * P + G];
                const bool bad = tl[3] != 0u;
                bad_any |= bad ? ABFT_EB_BAD_INDEX : 0;
                float a = as_f32(tl[0]), c = as_f32(tl[1]);
                if (kWeighted) {
                    a = wreg[k] * a;
                    c = wreg[k] * c;
                }
                a = bad ? 0.0f : a;
                c = bad ? 0.0f : c;
                v4u out;
                out[0] = __builtin_bit_cast(unsigned int, a);
                out[1] = __builtin_bit_cast(unsigned int, c);
                out[2] = out[3] = 0u;
                if (kCheck) {
                    // Eq. 4, the term of one pooled row: scale * C_T + d * bias, rounded once (both products
                    // are exact in binary64)
                    const double t = fma((double)a, (double)(bad ? 0 : (int32_t)tl[2]), (double)D * (double)c);
                    const unsigned long long tb = __builtin_bit_cast(unsigned long long, t);
                    out[2] = (unsigned int)tb;
                    out[3] = (unsigned int)(tb >> 32);
                }
                s_rec[r * P + G] = out;
            }
        }
        if (bad_any) atomicOr(&s_flag, bad_any);
        __syncthreads();
        // pooling, rows in index order
        if (col_thread) {
#pragma unroll 8
            for (int r = 0; r < n; ++r) {
                const float a = row_scale(r);
                const uint8_t* codes = s_bytes + r * REC + tid * BPT;
                unsigned int cw = BPT == 1 ? (unsigned int)*codes : (unsigned int)*reinterpret_cast<const uint16_t*>(codes);
#pragma unroll
                for (int k = 0; k < CPL; ++k) acc[k] = __builtin_fmaf(a, (float)((cw >> (BITS * k)) & ((1u << BITS) - 1u)), acc[k]);
            }
        }
        if (beta_wave) {
#pragma unroll 8
            for (int r = 0; r < n; ++r) beta_sum = beta_sum + row_bias(r);
        }
        if (kCheck && cs_wave) {
            // CSum: the lanes of this wavefront take every 64th row each and are added up at the end.  (The
            // terms are exact to their one rounding; only the order of their sum differs from index order,
            // by at most n * 2^-53 * sum |term|, eleven decimal orders below the bound of the comparison.
            // Walking them in index order is a chain of dependent binary64 additions that takes longer
            // than the pooling it runs beside.)
            for (int r = lane; r < n; r += 64) cs = cs + row_term(r);
        }
    }

    if (beta_wave && lane == 0) s_beta = beta_sum;
    if (kCheck && cs_wave) {
        cs = wave_sum(cs);
        if (lane == 0) s_cs = cs;
    }
    __syncthreads();
    const float beta = s_beta;
    double rs = 0.0;
    if (col_thread) {
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const float v = acc[k] + beta;
            p.R[bag * p.ldr + tid * CPL + k] = v;
            if (kCheck) rs += (double)v;
        }
    }
    if (kCheck) {
        rs = wave_sum(rs);
        if (lane == 0) s_rs[wave] = rs;
        __syncthreads();
        if (tid == 0) {
            const double total = (s_rs[0] + s_rs[1]) + (s_rs[2] + s_rs[3]);
            p.flags[bag] = s_flag | compare_sums(total, s_cs, p.bound);
            if (p.rsum) p.rsum[bag] = total;
            if (p.csum) p.csum[bag] = s_cs;
        }
    } else if (p.flags && tid == 0) {
        p.flags[bag] = s_flag;
    }
}

template <int G, int BITS>
hipError_t launch_g(bool group, bool check, bool weighted, const EbParams& p, hipStream_t s) {
    // one set of rows per lane only where the rows are wide and the launch has at least four wavefronts
    // per SIMD (measured at 16384 and 65536 lookups of 256 columns: 2 and 4 % faster than two sets;
    // everywhere else two sets are faster, by up to 30 % at 4096 lookups)
    const bool two_sets = G < 16 || p.n_bags * G < (int64_t)4096 * 64;
#define ABFT_EB_LAUNCH(CK, WT)                                                                                     \
    do {                                                                                                           \
        if (group) eb_group_kernel<G, BITS, CK, WT><<<dim3((unsigned)p.n_bags), dim3(256), 0, s>>>(p);             \
        else if (two_sets) eb_batch_kernel<G, BITS, CK, WT, true><<<dim3((unsigned)((p.n_bags * G + 255) / 256)), dim3(256), 0, s>>>(p); \
        else eb_batch_kernel<G, BITS, CK, WT, (G < 16)><<<dim3((unsigned)((p.n_bags * G + 255) / 256)), dim3(256), 0, s>>>(p); \
        return hipGetLastError();                                                                                  \
    } while (0)
    if (check && weighted) ABFT_EB_LAUNCH(true, true);
    if (check) ABFT_EB_LAUNCH(true, false);
    if (weighted) ABFT_EB_LAUNCH(false, true);
    ABFT_EB_LAUNCH(false, false);
#undef ABFT_EB_LAUNCH
}

template <int BITS>
hipError_t launch_bits(int code_bytes, bool group, bool check, bool weighted, const EbParams& p, hipStream_t s) {
    switch (code_bytes) {
        case 16: return launch_g<1, BITS>(group, check, weighted, p, s);
        case 32: return launch_g<2, BITS>(group, check, weighted, p, s);
        case 64: return launch_g<4, BITS>(group, check, weighted, p, s);
        case 128: return launch_g<8, BITS>(group, check, weighted, p, s);
        case 256: return launch_g<16, BITS>(group, check, weighted, p, s);
        case 512: return launch_g<32, BITS>(group, check, weighted, p, s);
    }
    return hipErrorNotSupported;
}

hipError_t launch_eb(int code_bytes, int bits, bool group, bool check, bool weighted, const EbParams& p, hipStream_t s) {
    return bits == 4 ? launch_bits<4>(code_bytes, group, check, weighted, p, s)
                     : launch_bits<8>(code_bytes, group, check, weighted, p, s);
}

// ---------------------------------------------------------------------------------------------
// Table build (Section V: row sums computed once), and the small helpers.
// One thread per 16-byte piece of a record; the thread of the tail piece sums the row's codes.
__global__ __launch_bounds__(256) void eb_pack_kernel(const uint8_t* T, int64_t ldt, const float* scale, const float* bias,
                                                      int64_t rows, int code_bytes, int bits, uint8_t* rec, int64_t stride) {
    const int P = code_bytes / 16 + 1;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = t / P;
    const int pc = (int)(t - row * P);
    if (row >= rows) return;
    const uint8_t* src = T + row * ldt;
    v4u out;
    if (pc < P - 1) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            unsigned int x = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) x |= (unsigned int)src[pc * 16 + 4 * w + b] << (8 * b);
            out[w] = x;
        }
    } else {
        int32_t sum = 0;
        for (int j = 0; j < code_bytes; ++j) sum += bits == 8 ? (int)src[j] : (int)(src[j] & 15) + (int)(src[j] >> 4);
        out[0] = __builtin_bit_cast(unsigned int, scale[row]);
        out[1] = __builtin_bit_cast(unsigned int, bias[row]);
        out[2] = (unsigned int)sum;
        out[3] = 0u;
    }
    *reinterpret_cast<v4u*>(rec + row * stride + pc * 16) = out;
}

__global__ __launch_bounds__(256) void eb_get_rowsums_kernel(const uint8_t* rec, int64_t stride, int64_t rows, int code_bytes, int32_t* C_T) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row < rows) C_T[row] = *reinterpret_cast<const int32_t*>(rec + row * stride + code_bytes + 8);
}

__global__ void eb_flip_kernel(uint8_t* rec, int64_t off, int bit) {
    if (threadIdx.x == 0 && blockIdx.x == 0) rec[off] = (uint8_t)(rec[off] ^ (1u << bit));
}

}  // namespace
}  // namespace abft

#define HIP_TRY(expr)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) return abft::set_error(ABFT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

extern "C" {

int abft_eb_pack_rowsum(const uint8_t* T, int64_t ldt, const float* scale, const float* bias, int64_t rows, int d,
                        unsigned flags, void* stream, abft_eb_table** out) {
    if (!T || !scale || !bias || !out) return abft::set_error(ABFT_EINVAL, "abft_eb_pack_rowsum: null pointer");
    if (rows < 1) return abft::set_error(ABFT_EINVAL, "abft_eb_pack_rowsum: rows=%lld must be >= 1", (long long)rows);
    if (flags & ~(ABFT_EB_PACK_LINE_ALIGNED | ABFT_EB_PACK_INT4)) return abft::set_error(ABFT_EINVAL, "abft_eb_pack_rowsum: unknown flag bits %#x", flags);
    const int bits = (flags & ABFT_EB_PACK_INT4) ? 4 : 8;
    const int code_bytes = d > 0 && d <= 4096 && (d * bits) % 8 == 0 ? d * bits / 8 : 0;
    if (code_bytes != 16 && code_bytes != 32 && code_bytes != 64 && code_bytes != 128 && code_bytes != 256 && code_bytes != 512)
        return abft::set_error(ABFT_EUNSUPPORTED, "abft_eb_pack_rowsum: d=%d with %d-bit codes (supported: rows of 16, 32, 64, 128, 256 or 512 bytes)", d, bits);
    if (ldt < code_bytes) return abft::set_error(ABFT_EINVAL, "abft_eb_pack_rowsum: ldt=%lld smaller than a row of %d bytes", (long long)ldt, code_bytes);
    // line-aligned: records of up to 128 bytes get a power-of-two stride, so none of them straddles a 128-byte line
    int64_t stride = code_bytes + 16;
    if ((flags & ABFT_EB_PACK_LINE_ALIGNED) && stride <= 128) stride = stride <= 32 ? 32 : (stride <= 64 ? 64 : 128);
    const int64_t pieces = rows * (code_bytes / 16 + 1);
    if ((pieces + 255) / 256 > 0x7fffffffll) return abft::set_error(ABFT_EUNSUPPORTED, "abft_eb_pack_rowsum: table too large");
    abft_eb_table* h = new (std::nothrow) abft_eb_table();
    if (!h) return abft::set_error(ABFT_EHIP, "abft_eb_pack_rowsum: out of host memory");
    std::memset(h, 0, sizeof *h);
    h->rows = rows;
    h->d = d;
    h->bits = bits;
    h->code_bytes = code_bytes;
    h->stride = stride;
    hipError_t e = hipGetDevice(&h->device);
    if (e == hipSuccess) e = hipMalloc(&h->rec, (size_t)rows * (size_t)stride);
    if (e == hipSuccess) {
        abft::eb_pack_kernel<<<dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
            T, ldt, scale, bias, rows, code_bytes, bits, h->rec, stride);
        e = hipGetLastError();
    }
    if (e != hipSuccess) {
        (void)hipFree(h->rec);
        delete h;
        return abft::set_error(ABFT_EHIP, "abft_eb_pack_rowsum: %s", hipGetErrorString(e));
    }
    *out = h;
    return ABFT_OK;
}

int abft_eb_table_dims(const abft_eb_table* Tp, int64_t* rows, int* d, int* record_bytes, int* bits) {
    if (!Tp) return abft::set_error(ABFT_EINVAL, "abft_eb_table_dims: null handle");
    if (rows) *rows = Tp->rows;
    if (d) *d = Tp->d;
    if (record_bytes) *record_bytes = (int)Tp->stride;
    if (bits) *bits = Tp->bits;
    return ABFT_OK;
}

int abft_eb_table_get_rowsums(const abft_eb_table* Tp, int32_t* C_T, void* stream) {
    if (!Tp || !C_T) return abft::set_error(ABFT_EINVAL, "abft_eb_table_get_rowsums: null pointer");
    abft::eb_get_rowsums_kernel<<<dim3((unsigned)((Tp->rows + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
        Tp->rec, Tp->stride, Tp->rows, Tp->code_bytes, C_T);
    HIP_TRY(hipGetLastError());
    return ABFT_OK;
}

int abft_eb_table_flip_bit(abft_eb_table* Tp, int64_t row, int col, int bit, void* stream) {
    if (!Tp) return abft::set_error(ABFT_EINVAL, "abft_eb_table_flip_bit: null handle");
    if (row < 0 || row >= Tp->rows || col < 0 || col >= Tp->d || bit < 0 || bit >= Tp->bits)
        return abft::set_error(ABFT_EINVAL, "abft_eb_table_flip_bit: row=%lld col=%d bit=%d outside the table", (long long)row, col, bit);
    // a 4-bit code of an odd column sits in the high half of its byte
    const int64_t off = row * Tp->stride + (Tp->bits == 8 ? col : col / 2);
    const int pos = Tp->bits == 8 ? bit : bit + 4 * (col & 1);
    abft::eb_flip_kernel<<<dim3(1), dim3(64), 0, (hipStream_t)stream>>>(Tp->rec, off, pos);
    HIP_TRY(hipGetLastError());
    return ABFT_OK;
}

void abft_eb_table_destroy(abft_eb_table* Tp) {
    if (!Tp) return;
    (void)hipFree(Tp->rec);
    delete Tp;
}

int abft_eb_u8_checked(const abft_eb_table* Tp, const int64_t* indices, int64_t n_indices, const int64_t* offsets,
                       int64_t n_bags, const float* weights, float* R, int64_t ldr, int32_t* bag_flags,
                       double* rsum, double* csum, double rel_bound, unsigned flags, void* stream) {
    const char* fn = "abft_eb_u8_checked";
    if (!Tp || !offsets) return abft::set_error(ABFT_EINVAL, "%s: null pointer", fn);
    if (n_indices < 0 || n_bags < 0) return abft::set_error(ABFT_EINVAL, "%s: negative count", fn);
    if (n_bags == 0) return ABFT_OK;  // nothing to pool, nothing is written
    if (!R) return abft::set_error(ABFT_EINVAL, "%s: null pointer", fn);
    if (n_indices > 0 && !indices) return abft::set_error(ABFT_EINVAL, "%s: null indices", fn);
    if (flags & ~(ABFT_EB_NOCHECK | ABFT_EB_VARIANT_MASK)) return abft::set_error(ABFT_EINVAL, "%s: unknown flag bits %#x", fn, flags);
    const bool check = (flags & ABFT_EB_NOCHECK) == 0;
    if (check && !bag_flags) return abft::set_error(ABFT_EINVAL, "%s: bag_flags is required unless ABFT_EB_NOCHECK", fn);
    if (check && !(rel_bound >= 0.0)) return abft::set_error(ABFT_EINVAL, "%s: rel_bound must be >= 0", fn);
    if (ldr < Tp->d || ldr % 4 != 0 || (reinterpret_cast<uintptr_t>(R) & 15) != 0)
        return abft::set_error(ABFT_EINVAL, "%s: R needs ldr >= d, ldr a multiple of 4 and 16-byte alignment", fn);
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != Tp->device)
        return abft::set_error(ABFT_EINVAL, "%s: the table lives on device %d, the current device is %d", fn, Tp->device, dev);
    const unsigned variant = flags & ABFT_EB_VARIANT_MASK;
    if (variant != 0 && variant != ABFT_EB_VARIANT_BATCH && variant != ABFT_EB_VARIANT_GROUP)
        return abft::set_error(ABFT_EINVAL, "%s: unknown variant %#x", fn, variant);
    const int G = Tp->code_bytes / 16;
    if (n_bags > 0x7fffffffll || (n_bags * G + 255) / 256 > 0x7fffffffll)
        return abft::set_error(ABFT_EUNSUPPORTED, "%s: n_bags=%lld too large for one launch", fn, (long long)n_bags);
    // The batch kernel needs enough lookups to fill the chip with lanes; below that one workgroup per lookup
    // keeps more bytes in flight.  Crossovers measured with 100 rows per lookup on a 2 GiB table, checked
    // (code bytes per row: lookups): 16: between 32768 and 65536; 32: 32768, within 2 % of each other
    // beyond; 64 and 128: the group kernel still ahead by 1 % at 65536 and 131072; 256: between 6144 and
    // 8192 (7 % either way); 512: group ahead by 4 % at 8192.
    bool group = n_bags < abft::eb_batch_min_lookups(G);
    if (variant == ABFT_EB_VARIANT_BATCH) group = false;
    if (variant == ABFT_EB_VARIANT_GROUP) group = true;
    abft::EbParams p;
    p.tab = Tp->rec;
    p.stride = Tp->stride;
    p.rows = Tp->rows;
    p.indices = indices;
    p.n_indices = n_indices;
    p.offsets = offsets;
    p.n_bags = n_bags;
    p.weights = weights;
    p.R = R;
    p.ldr = ldr;
    p.flags = bag_flags;
    p.rsum = check ? rsum : nullptr;
    p.csum = check ? csum : nullptr;
    p.bound = rel_bound;
    HIP_TRY(abft::launch_eb(Tp->code_bytes, Tp->bits, group, check, weights != nullptr, p, (hipStream_t)stream));
    return ABFT_OK;
}

}  // extern "C"
