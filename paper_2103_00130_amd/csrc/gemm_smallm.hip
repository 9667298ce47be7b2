// Streaming checked u8 x s8 -> s32 GEMM for M <= 64 (tall-skinny, batch-of-requests shapes).
//
// Algorithm 1 of arXiv 2103.00130 (product with the encoded B, row sums, comparison) for the
// shapes where the weight matrix is read once and barely reused: the kernel is bound by
// streaming the packed B from HBM, so the design goal is bytes in flight, not MFMA rate.
//
//  * One workgroup owns 16 columns for the whole K range; its four wavefronts take the
//    k-blocks kb = wave, wave+4, ... and issue their loads in batches, two batches in flight,
//    so that the grid as a whole keeps the entire weight matrix in flight.  No LDS staging:
//    a 16x16x64 int8 MFMA B operand is read straight from the packed layout (four 256-byte
//    runs per instruction), the A operand straight from A (it is small and lives in L2).
//  * u8 -> s8 by XOR 0x80 on the A operand, +128 * (column sum of the streamed B bytes) added
//    back; the checksum column S_B rides as four base-256 digit columns on a second MFMA; the
//    column blocks split its K range between them.
//  * The four partial accumulators meet in LDS; wavefront 0 adds them, forms the row sums with
//    DPP row reductions, stores C, and then adds (row sum - checksum) per row into 64-bit
//    workspace words that also count arrivals (returned integer atomics, a few dozen arrivals
//    per word at most): whoever completes a row's word writes its flag, whoever completes the
//    count of finished rows writes errCount, and each clears what it completed.  No workgroup
//    waits for another and there is no closing pass.
#include "../../include/abft_gemm.h"
#include "abft_internal.h"

namespace abft {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
constexpr int kOutC = 1, kOutQ = 2;
constexpr int kSmallMWideN = 8192;   // from this width on a workgroup owns 32 columns (M <= 32): at least 256 workgroups remain (with fewer, 16 x 4096 x 2048 runs in 5.6 us instead of 4.7)

// sum over the 16 lanes of a DPP row; every lane of the row ends up with the total
__device__ inline uint32_t row_sum16(uint32_t s) {
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0x141, 0xF, 0xF, true);  // row_half_mirror
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0x140, 0xF, 0xF, true);  // row_mirror
    return s;
}

// v mod 127 in [0,126] for |v| < 2^59 (2^28 is 1 modulo 127, so the two parts of v = hi * 2^28 + lo may be added)
__device__ inline int32_t floor_mod127(long long v) {
    const int32_t x = (int32_t)(v >> 28) + (int32_t)(v & 0x0FFFFFFF);
    const int32_t r = x % 127;
    return r < 0 ? r + 127 : r;
}

// RB = 16-row blocks of A (M <= 16*RB); NCB = blocks of 16 columns per workgroup.  With NCB = 2 a workgroup owns a
// whole 32-column unit of the packed weight, with NCB = 4 two neighbouring units: every k-block it reads is 2 or
// 4 KiB of contiguous memory instead of every other 256 bytes of it, and one A operand serves two or four matrix
// instructions (wide weights, where the column blocks alone fill the chip many times over; measured at M = 16 on
// 16384 x 32768 int8: 0.49 of the HBM peak with NCB = 1, 0.64 with 2, 0.70 with 4).
template <int RB, int NCB, bool kCheck, int kOut>
__global__ __launch_bounds__(256) void gemm_smallm_kernel(const GemmParams p, const int n_blocks) {
    constexpr int BATCH = (RB == 1 ? 8 : 4) / NCB > 0 ? (RB == 1 ? 8 : 4) / NCB : 1;  // k-blocks per wave per batch of loads
    constexpr bool kWantC = (kOut & kOutC) != 0, kWantQ = (kOut & kOutQ) != 0;
    __shared__ v4i s_acc[3][NCB][RB][64];
    __shared__ v4i s_chk[3][RB][64];
    __shared__ uint32_t s_bsum[3][NCB][64];
    __shared__ uint32_t s_d[64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cb = blockIdx.x, col0 = cb * 16 * NCB;
    const int KB = p.KB;
    const int lcol = lane & 15, lkg = lane >> 4;

    // B operand of k-block kb: unit of col0, columns 16*half .. +15, k-group lkg
    const int8_t* const b_src = p.packed + packed_unit_offset(col0 / kTileN, 0, (col0 % kTileN) / kUnitN, KB) +
                                (lkg * kUnitN + (col0 % kUnitN) + lcol) * 16;
    constexpr int64_t B_KB_STRIDE = (int64_t)kUnitsPerTile * kUnitBytes;
    // A operand of row block rb: row rb*16 + lcol (clamped), k-group lkg
    const uint8_t* a_row[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) a_row[rb] = p.A + (int64_t)min(rb * 16 + lcol, p.M - 1) * p.lda;
    // this column block's share of the checksum product's K range
    const int lo = share_begin(cb, p.share_q, p.share_r), hi = share_begin(cb + 1, p.share_q, p.share_r);

    // sum_k S_B[k] for the first column block's share of the check, fetched ahead of its use at the very end
    const int32_t total_sb = (kCheck && cb == 0) ? *p.total : 0;

    v4i acc[NCB][RB], cacc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        cacc[rb] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < NCB; ++c) acc[c][rb] = v4i{0, 0, 0, 0};
    }
    uint32_t bsum[NCB];
#pragma unroll
    for (int c = 0; c < NCB; ++c) bsum[c] = 0;

    v4i fb[2][BATCH][NCB], fa[2][BATCH][RB], fl[2][BATCH];
    auto issue = [&](int kb0, int s) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int kb = kb0 + 4 * u;
            const int kbc = min(kb, KB - 1);
            // a k-block past the end is fetched from the last one and zeroed below
#pragma unroll
            for (int c = 0; c < NCB; ++c)   // the next 16 columns of a unit lie 256 bytes further on, the next unit 2 KiB
                fb[s][u][c] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(b_src + (int64_t)kbc * B_KB_STRIDE + (c >> 1) * kUnitBytes + (c & 1) * 256));
            const int k = min(kbc * 64 + lkg * 16, p.K - 16);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) fa[s][u][rb] = *reinterpret_cast<const v4i*>(a_row[rb] + k);
            if (kCheck) {
                fl[s][u] = v4i{0, 0, 0, 0};
                if (kb >= lo && kb < hi && lcol < kLimbs)
                    fl[s][u] = *reinterpret_cast<const v4i*>(p.limbs + ((((int64_t)kb * 4 + lkg) * kLimbs + lcol) << 4));
            }
        }
    };
    auto consume = [&](int kb0, int s) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int kb = kb0 + 4 * u;
            v4i b[NCB];
#pragma unroll
            for (int c = 0; c < NCB; ++c) {
                b[c] = fb[s][u][c];
                if (kb >= KB) b[c] = v4i{0, 0, 0, 0};
                // bytes of B as biased uint8, summed four at a time; the bias comes off at the end
                bsum[c] = __builtin_amdgcn_sad_u8((uint32_t)b[c].x ^ 0x80808080u, 0u, bsum[c]);
                bsum[c] = __builtin_amdgcn_sad_u8((uint32_t)b[c].y ^ 0x80808080u, 0u, bsum[c]);
                bsum[c] = __builtin_amdgcn_sad_u8((uint32_t)b[c].z ^ 0x80808080u, 0u, bsum[c]);
                bsum[c] = __builtin_amdgcn_sad_u8((uint32_t)b[c].w ^ 0x80808080u, 0u, bsum[c]);
            }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const v4i a = fa[s][u][rb] ^ (int)0x80808080;
#pragma unroll
                for (int c = 0; c < NCB; ++c) acc[c][rb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[c], acc[c][rb], 0, 0, 0);
                if (kCheck) cacc[rb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, fl[s][u], cacc[rb], 0, 0, 0);
            }
        }
    };

    // k-blocks of this wave: wave, wave+4, ...; the same number of batches for every wave
    const int per_wave = (KB + 3) / 4;
    const int n_batches = (per_wave + BATCH - 1) / BATCH;
    issue(wave, 0);
    for (int bt = 0; bt < n_batches; bt += 2) {
        if (bt + 1 < n_batches) issue(wave + 4 * BATCH * (bt + 1), 1);
        consume(wave + 4 * BATCH * bt, 0);
        if (bt + 1 < n_batches) {
            if (bt + 2 < n_batches) issue(wave + 4 * BATCH * (bt + 2), 0);
            consume(wave + 4 * BATCH * (bt + 1), 1);
        }
    }

    // ---- the four partial results meet in wavefront 0 --------------------------------
    if (wave > 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
            for (int c = 0; c < NCB; ++c) s_acc[wave - 1][c][rb][lane] = acc[c][rb];
            if (kCheck) s_chk[wave - 1][rb][lane] = cacc[rb];
        }
#pragma unroll
        for (int c = 0; c < NCB; ++c) s_bsum[wave - 1][c][lane] = bsum[c];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                for (int c = 0; c < NCB; ++c) acc[c][rb] += s_acc[w][c][rb][lane];
                if (kCheck) cacc[rb] += s_chk[w][rb][lane];
            }
#pragma unroll
            for (int c = 0; c < NCB; ++c) bsum[c] += s_bsum[w][c][lane];
        }
        // every lane summed 16 biased bytes per k-block slot; 4 waves x n_batches x BATCH slots x 4 k-groups
        const uint32_t bias = 128u * 16u * 4u * 4u * (uint32_t)(n_batches * BATCH);
#pragma unroll
        for (int c = 0; c < NCB; ++c) {
            // column sum of the streamed B for column lcol: the four k-groups sit in lanes lcol + 16*g
            // (row swap and half swap: both return {own, partner} in an order that depends on the lane)
            const auto r16 = __builtin_amdgcn_permlane16_swap(bsum[c], bsum[c], false, false);
            bsum[c] = r16[0] + r16[1];
            const auto r32 = __builtin_amdgcn_permlane32_swap(bsum[c], bsum[c], false, false);
            bsum[c] = r32[0] + r32[1];
            const int32_t cs128 = 128 * (int32_t)(bsum[c] - bias);
            // accumulator layout of the 16x16 MFMA: lane l, element e is row 4*(l/16) + e, column l%16
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[c][rb][e] += cs128;
        }

        if (p.n_inj > 0) {
            // simulated faults in the 32-bit intermediate (test hook): XOR before the row sums
            const abft_inject_t* inj = reinterpret_cast<const abft_inject_t*>(p.inj);
            for (int n = 0; n < p.n_inj; ++n) {
                const int r = inj[n].row, c = inj[n].col - col0;
                if (r < 0 || r >= p.M || r >= 16 * RB || c < 0 || c >= 16 * NCB || inj[n].col >= p.N) continue;
                const bool mine = (lcol == (c & 15)) && (lkg == ((r & 15) >> 2));
#pragma unroll
                for (int cc = 0; cc < NCB; ++cc)
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (mine && cc == (c >> 4) && rb == (r >> 4) && e == (r & 3)) acc[cc][rb][e] ^= (int)inj[n].xor_mask;
            }
        }

        // stores first (they need no answer), then the check, whose atomics wait for theirs;
        // per (rb, e) one store instruction covers 4 rows x 16 columns
#pragma unroll
        for (int c = 0; c < NCB; ++c) {
            const int col = col0 + c * 16 + lcol;
            RequantCol rqc;   // this lane's column, fetched once
            rqc.sub = 0;
            rqc.mult = 0.0f;
            if (kWantQ && col < p.N) rqc = requant_col(p.colsum[col], col, p.rq);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = rb * 16 + 4 * lkg + e;
                    if (row < p.M && col < p.N) {
                        if (kWantC) p.C[(int64_t)row * p.ldc + col] = acc[c][rb][e];
                        if (kWantQ) p.Cq[(int64_t)row * p.ldcq + col] = requant_with(acc[c][rb][e], rqc, p.rq.zC);
                    }
                }
        }
        if (kCheck) {
            const bool mod127 = p.mod127 != 0;
            const int slot = cb & (kSmallMSlots - 1);
            const uint32_t total128 = 128u * (uint32_t)total_sb;  // sum_k 128*S_B[k], once per row (first column block)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // (Algorithm 1 as printed, p.mod127: the entries are exact 32-bit values, K <= 65536, and are
                    // summed as residues; the one live digit column holds rowSum, so its product is exact too)
                    uint32_t mine = 0;   // this lane's entries of the row (residues of them under the printed modulus)
#pragma unroll
                    for (int c = 0; c < NCB; ++c)
                        mine += mod127 ? (uint32_t)floor_mod127((long long)acc[c][rb][e]) : (uint32_t)acc[c][rb][e];
                    const uint32_t rs = row_sum16(mine);
                    uint32_t ck = lcol < kLimbs ? ((uint32_t)cacc[rb][e] << (8 * lcol)) : 0u;
                    ck += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)ck, 0xB1, 0xF, 0xF, true);
                    ck += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)ck, 0x4E, 0xF, 0xF, true);
                    const int row = rb * 16 + 4 * lkg + e;
                    if (lcol == 0)
                        s_d[row] = mod127 ? (uint32_t)floor_mod127((long long)rs - (long long)(int32_t)ck - 128ll * (long long)total_sb)
                                          : rs - ck - total128;
                }
            // One row per lane.  The row's difference climbs workspace words, each a 64-bit
            // (value << 32 | arrivals) taken with one returned atomic.  With more than 32 column
            // blocks the first word is that of (slot, row), shared by the blocks of one slot, whose
            // last arrival carries the slot's sum on; the next is the word of the row, where the last
            // arrival has the complete difference and writes the flag.  The rows a wavefront finishes
            // are counted with one atomic on the word of finished rows, whose last arrival writes
            // errCount.  Every word is cleared by the arrival that completes it.  No word sees more
            // than a few dozen arrivals, and nobody waits for anybody.
            bool fin = false, bad = false;
            if (lane < 16 * RB && lane < p.M) {
                unsigned long long* const w_slot =
                    reinterpret_cast<unsigned long long*>(p.ws + kWsHeaderInts) + slot * kSmallMRows + lane;
                unsigned long long* const w_row =
                    reinterpret_cast<unsigned long long*>(p.ws + kWsHeaderInts) + kSmallMSlots * kSmallMRows + lane;
                uint32_t t = s_d[lane], n_row = (uint32_t)n_blocks;
                bool go = true;
                if (n_blocks > kSmallMSlots) {
                    const uint32_t n_slot = ((uint32_t)n_blocks - (uint32_t)slot + kSmallMSlots - 1) / kSmallMSlots;
                    const unsigned long long old = __hip_atomic_fetch_add(w_slot, ((unsigned long long)t << 32) | 1ull,
                                                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    go = (uint32_t)old == n_slot - 1u;
                    if (go) {
                        t += (uint32_t)(old >> 32);
                        __hip_atomic_store(w_slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    n_row = (uint32_t)kSmallMSlots;
                }
                if (n_blocks == 1) {
                    // a single column block holds the whole row: nothing crosses workgroups
                    bad = mod127 ? (t % 127u != 0u) : (t != 0u);
                    p.row_flags[lane] = (int32_t)bad;
                    fin = true;
                } else if (go) {
                    const unsigned long long old = __hip_atomic_fetch_add(w_row, ((unsigned long long)t << 32) | 1ull,
                                                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((uint32_t)old == n_row - 1u) {
                        const uint32_t diff = (uint32_t)(old >> 32) + t;
                        bad = mod127 ? (diff % 127u != 0u) : (diff != 0u);
                        __hip_atomic_store(w_row, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        p.row_flags[lane] = (int32_t)bad;
                        fin = true;
                    }
                }
            }
            // errCount: not asked for / added to by the wavefronts that found corrupted rows (no return value,
            // nobody waits) / overwritten by the report that brings the count of finished rows to M
            const unsigned long long fin_mask = __ballot(fin), bad_mask = __ballot(fin && bad);
            if (p.err_count == nullptr) {
            } else if (p.err_accumulate) {
                if (bad_mask != 0ull && lane == __builtin_ctzll(bad_mask))
                    __hip_atomic_fetch_add(p.err_count, (int32_t)__builtin_popcountll(bad_mask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (fin_mask != 0ull && lane == __builtin_ctzll(fin_mask)) {
                unsigned long long* const w_done = reinterpret_cast<unsigned long long*>(p.ws + kWsDoneWord);
                const uint32_t n_fin = (uint32_t)__builtin_popcountll(fin_mask), n_bad = (uint32_t)__builtin_popcountll(bad_mask);
                const unsigned long long old = __hip_atomic_fetch_add(w_done, ((unsigned long long)n_bad << 32) | n_fin,
                                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((uint32_t)old + n_fin == (uint32_t)p.M) {
                    *p.err_count = (int32_t)((uint32_t)(old >> 32) + n_bad);
                    __hip_atomic_store(w_done, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

template <int RB, int NCB>
hipError_t launch_rb(bool check, bool want_c, bool want_q, const GemmParams& p_in, hipStream_t s) {
    GemmParams p = p_in;
    const int n_blocks = (p.N + 16 * NCB - 1) / (16 * NCB);
    p.share_q = p.KB / n_blocks;   // k-blocks of the checksum product per column block
    p.share_r = p.KB % n_blocks;
    const dim3 grid((unsigned)n_blocks), block(256);
#define ABFT_LAUNCH(CK, OUT)                                                         \
    do {                                                                             \
        gemm_smallm_kernel<RB, NCB, CK, OUT><<<grid, block, 0, s>>>(p, n_blocks);    \
        return hipGetLastError();                                                    \
    } while (0)
#define ABFT_OUT(CK)                                          \
    do {                                                      \
        if (want_c && want_q) ABFT_LAUNCH(CK, kOutC | kOutQ); \
        if (want_c) ABFT_LAUNCH(CK, kOutC);                   \
        ABFT_LAUNCH(CK, kOutQ);                               \
    } while (0)
    if (check) ABFT_OUT(true);
    ABFT_OUT(false);
#undef ABFT_OUT
#undef ABFT_LAUNCH
}

}  // namespace

hipError_t launch_gemm_smallm(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    if (p.M > 64 || !p.a_vec_ok || p.K % 16 != 0) return hipErrorNotSupported;
    // whole 32-column units per workgroup once the 16-column blocks alone would fill the chip at least twice
    const bool wide = p.N >= kSmallMWideN;
    if (p.M <= 16 && p.N >= 2 * kSmallMWideN) return launch_rb<1, 4>(check, want_c, want_q, p, s);
    if (p.M <= 16) return wide ? launch_rb<1, 2>(check, want_c, want_q, p, s) : launch_rb<1, 1>(check, want_c, want_q, p, s);
    if (p.M <= 32) return wide ? launch_rb<2, 2>(check, want_c, want_q, p, s) : launch_rb<2, 1>(check, want_c, want_q, p, s);
    return launch_rb<4, 1>(check, want_c, want_q, p, s);
}

}  // namespace abft
