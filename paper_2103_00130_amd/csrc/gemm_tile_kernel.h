// Checked u8 x s8 -> s32 GEMM, LDS-tiled int8-MFMA kernel for gfx950 (template).
//
// Algorithm 1 of arXiv 2103.00130 from the product line on: C_temp = A * [B | S_B]
// in ONE pass over A (Section IV-A-3, the checksum rides the level-3 product), then
// tSum per row, the comparison of Eq. 2b and errCount, then (optionally) the
// requantization of Section III-B, which never sees the checksum column
// (Section IV-B: the check reads the 32-bit values).
//
// How the pieces map to the hardware
//  * A is uint8 but the int8 matrix cores multiply signed by signed: A is staged as
//    a' = a XOR 0x80 (= a - 128) and 128 * (column sum of the B bytes streamed) is
//    added back in the epilogue, which is exact modulo 2^32.
//  * S_B[k] is an int32.  It enters the same MFMA pipeline as four signed base-256
//    digit columns; the epilogue recombines the four partial products with shifts.
//    Everything is a ring homomorphism mod 2^32, so the result equals A * S_B exactly.
//  * The checksum columns are shared by the whole matrix row, so the tile columns of
//    the grid split the K range of the checksum product between them (tile column c
//    takes the k-blocks with kb % tiles_n == c, which it streams through LDS anyway).
//    Each workgroup adds (partial row sum - partial checksum) per row into a
//    workspace with integer atomics; the last workgroup to arrive turns the sums
//    into flags.  Integer addition commutes, so the outcome does not depend on order.
//  * Software pipeline per k-block of 64: global loads run 1.5 iterations ahead into
//    two register sets, are staged to the other LDS buffer while the first half of
//    the MFMAs issues, and the fragments of the next half-step are read from LDS while
//    the current half-step's MFMAs run; one barrier per k-block.
#pragma once
#include "../../include/abft_gemm.h"
#include <type_traits>

#include "abft_internal.h"

namespace abft {
namespace tile {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kOutC = 1, kOutQ = 2;

// LDS position of the 16-byte chunk (row r of the tile, k-group kg).  Rows are cut in
// blocks of 32; inside a block the four k-groups are 512-byte planes and plane kg is
// rotated by 4*kg slots so that the staging stores (4 consecutive lanes = 4 k-groups of
// one row) and the fragment loads (32 consecutive rows of one plane) both spread over
// the banks.
__device__ inline int a_lds_off(int r, int kg) {
    return (r >> 5) * 2048 + (kg * 32 + ((r + 4 * kg) & 31)) * 16;
}

// This is the general path: A may have any alignment, leading dimension and K; its
// chunks are assembled byte by byte.  Aligned problems take the kernel of
// gemm_tile_async.h instead.
template <int BM, int BN, int WGM, int WGN, bool kCheck, int kOut>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_tile_kernel(const GemmParams p, const int tiles_n) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 blocks per wave
    constexpr int A_CH = BM * 4 / NT, B_CH = BN * 4 / NT;
    constexpr int CB = (WTM / 16) / WGN;           // 16-row checksum blocks per wave
    constexpr bool kWantC = (kOut & kOutC) != 0, kWantQ = (kOut & kOutQ) != 0;
    static_assert(A_CH >= 1 && B_CH >= 1 && CB >= 1 && 4 * BN >= NT, "tile too small for the workgroup");
    static_assert((WTM / 16) % WGN == 0, "checksum rows must split evenly over the waves of a row");
    constexpr int A_BYTES = BM * 64, B_BYTES = BN * 64;

    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* const sA = smem;                  // [2][A_BYTES]
    uint8_t* const sB = smem + 2 * A_BYTES;    // [2][B_BYTES]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int tile_n = blockIdx.x % tiles_n, tile_m = blockIdx.x / tiles_n;
    const int row0 = tile_m * BM, col0 = tile_n * BN;
    const int KB = p.KB;

    // packed B: this tile's BN columns of k-block kb are BN*64 consecutive bytes
    constexpr int TILES_PER_NT = kTileN / BN;
    const int8_t* const b_tile =
        p.packed + packed_unit_offset(tile_n / TILES_PER_NT, 0, (tile_n % TILES_PER_NT) * (BN / 32), KB);
    constexpr int64_t B_KB_STRIDE = (int64_t)kUnitsPerTile * kUnitBytes;

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
    v4i cacc[CB];
#pragma unroll
    for (int i = 0; i < CB; ++i) cacc[i] = v4i{0, 0, 0, 0};

    // two register sets for the global loads in flight
    v4i ra[2][A_CH], rb[2][B_CH], rl[2];
    rl[0] = rl[1] = v4i{0, 0, 0, 0};
    // Column sums of the B bytes this workgroup actually streams, for the +128*colsum
    // add-back: taking them from the data in flight (not from the sums stored at pack
    // time) keeps C_temp = A*B exact for whatever B is in memory, faulty or not.
    int32_t bsum[B_CH];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) bsum[i] = 0;

    auto g_load = [&](int kb, int s) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int q = tid + NT * i;
            {
                const int r = q >> 2, kg = q & 3;
                const int grow = row0 + r, k0 = kb * 64 + kg * 16;
                v4i v = v4i{0, 0, 0, 0};
                if (grow < p.M && k0 < p.K) {
                    const uint8_t* src = p.A + (int64_t)grow * p.lda + k0;
                    const int nb = min(16, p.K - k0);
                    for (int b = 0; b < nb; ++b) {
                        const uint32_t sh = (uint32_t)src[b] << (8 * (b & 3));
                        if ((b >> 2) == 0) v.x |= (int)sh;
                        else if ((b >> 2) == 1) v.y |= (int)sh;
                        else if ((b >> 2) == 2) v.z |= (int)sh;
                        else v.w |= (int)sh;
                    }
                }
                ra[s][i] = v;
            }
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            const int q = tid + NT * i;
            rb[s][i] = *reinterpret_cast<const v4i*>(b_tile + (int64_t)kb * B_KB_STRIDE + q * 16);
        }
        if (kCheck) {
            rl[s] = v4i{0, 0, 0, 0};
            if ((kb % tiles_n) == tile_n && (lane & 15) < kLimbs)
                rl[s] = *reinterpret_cast<const v4i*>(p.limbs + (((int64_t)kb * 4 + (lane >> 4)) * kLimbs + (lane & 15)) * 16);
        }
    };
    auto stage = [&](int s, int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int q = tid + NT * i;
            *reinterpret_cast<v4i*>(sA + buf * A_BYTES + a_lds_off(q >> 2, q & 3)) = ra[s][i] ^ (int)0x80808080;
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            const int q = tid + NT * i;
            *reinterpret_cast<v4i*>(sB + buf * B_BYTES + q * 16) = rb[s][i];
            bsum[i] = __builtin_amdgcn_sdot4(rb[s][i].x, 0x01010101, bsum[i], false);
            bsum[i] = __builtin_amdgcn_sdot4(rb[s][i].y, 0x01010101, bsum[i], false);
            bsum[i] = __builtin_amdgcn_sdot4(rb[s][i].z, 0x01010101, bsum[i], false);
            bsum[i] = __builtin_amdgcn_sdot4(rb[s][i].w, 0x01010101, bsum[i], false);
        }
    };
    v4i fa[2][TM], fb[2][TN];
    auto read_frags = [&](int buf, int h, int f) {
        const uint8_t* a_cur = sA + buf * A_BYTES;
        const uint8_t* b_cur = sB + buf * B_BYTES;
        const int kg = 2 * h + (lane >> 5);
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[f][i] = *reinterpret_cast<const v4i*>(a_cur + a_lds_off(wm * WTM + i * 32 + (lane & 31), kg));
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[f][j] = *reinterpret_cast<const v4i*>(b_cur + (wn * TN + j) * 2048 + h * 1024 + lane * 16);
    };
    auto mma = [&](int f) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[f][i], fb[f][j], acc[i][j], 0, 0, 0);
    };

    v4i limb_cur = v4i{0, 0, 0, 0}, limb_nxt = v4i{0, 0, 0, 0};
    // s_waitcnt with only the LDS/scalar counter at zero (vmcnt and expcnt left open)
    auto wait_lds = [] { __builtin_amdgcn_s_waitcnt(0xC07F); };
    // One k-block.  CUR = kb & 1 picks the LDS buffer and, with it, the register set that
    // was loaded for kb+1; both are compile-time so that no register array is indexed at
    // run time.  LAST drops everything that prepares a following k-block.
    auto body = [&](int kb, auto cur_c, auto last_c) {
        constexpr int CUR = decltype(cur_c)::value;
        constexpr bool LAST = decltype(last_c)::value;
        // first half-step: fragments of the second half come in, the next tile goes to LDS
        read_frags(CUR, 1, 1);
        if (!LAST) {
            stage(CUR ^ 1, CUR ^ 1);
            limb_nxt = rl[CUR ^ 1];
        }
        mma(0);
#pragma unroll
        for (int g = 0; g < (TM + TN < 8 ? TM + TN : 8); ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
        }
        if (!LAST) {
#pragma unroll
            for (int g = 0; g < (A_CH + B_CH < 8 ? A_CH + B_CH : 8); ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);  // a few VALU (xor, dot4, addresses)
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // one LDS write
            }
        }
        if (kCheck && (kb % tiles_n) == tile_n) {
            const uint8_t* a_cur = sA + CUR * A_BYTES;
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                const int r = wm * WTM + (wn * CB + c) * 16 + (lane & 15);
                const v4i a = *reinterpret_cast<const v4i*>(a_cur + a_lds_off(r, lane >> 4));
                cacc[c] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, limb_cur, cacc[c], 0, 0, 0);
            }
        }
        limb_cur = limb_nxt;
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        // second half-step: the register set just staged is free for the loads of kb+3
        if (!LAST) {
            g_load(min(kb + 3, KB - 1), CUR ^ 1);
            read_frags(CUR ^ 1, 0, 0);
        }
        mma(1);
        if (!LAST) {
#pragma unroll
            for (int g = 0; g < (A_CH + B_CH < 8 ? A_CH + B_CH : 8); ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // one global load
            }
#pragma unroll
            for (int g = 0; g < (TM + TN < 8 ? TM + TN : 8); ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
            }
        }
        // the fragment reads have long landed behind the MFMAs: retire them here so that the
        // next half-step can issue its MFMAs without waiting on what it is about to enqueue
        wait_lds();
        __builtin_amdgcn_sched_barrier(0);
    };
    using c0 = std::integral_constant<int, 0>;
    using c1 = std::integral_constant<int, 1>;

    g_load(0, 0);
    g_load(min(1, KB - 1), 1);
    stage(0, 0);
    limb_cur = rl[0];
    __syncthreads();
    g_load(min(2, KB - 1), 0);
    read_frags(0, 0, 0);
    wait_lds();
    __builtin_amdgcn_sched_barrier(0);

    int kb = 0;
    for (; kb + 2 < KB; kb += 2) {
        body(kb, c0{}, std::false_type{});
        body(kb + 1, c1{}, std::false_type{});
    }
    if (kb + 1 < KB) {
        body(kb, c0{}, std::false_type{});
        body(kb + 1, c1{}, std::true_type{});
    } else {
        body(kb, c0{}, std::true_type{});
    }
    __syncthreads();

    // ---------------------------------- epilogue ----------------------------------
    // accumulator layout of the 32x32 MFMA: lane l, element e of block (i, j) is
    // row 8*(e/4) + 4*(l/32) + e%4, column l%32 of that block.
    const int lcol = lane & 31, lhalf = lane >> 5;
    // LDS is free now: [4][BN] column-sum parts, [WGN][BM] row-sum parts, [BM] checksum
    // parts, 4 control words.
    int32_t* const s_bs = reinterpret_cast<int32_t*>(smem);
    int32_t* const s_rs = s_bs + 4 * BN;
    int32_t* const s_ck = s_rs + WGN * BM;
    int* const s_ctl = s_ck + BM;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        const int q = tid + NT * i;  // chunk q of the tile: unit q/128, k-group (q/32)%4, column q%32
        s_bs[((q >> 5) & 3) * BN + (q >> 7) * 32 + (q & 31)] = bsum[i];
    }
    __syncthreads();
    int32_t cs[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int c = wn * WTN + j * 32 + lcol;
        cs[j] = s_bs[c] + s_bs[BN + c] + s_bs[2 * BN + c] + s_bs[3 * BN + c];
    }

    // C_temp values: undo the a - 128 shift
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] += 128 * cs[j];

    if (p.n_inj > 0) {
        // simulated faults in the 32-bit intermediate (test hook): XOR before the row sums
        const abft_inject_t* inj = reinterpret_cast<const abft_inject_t*>(p.inj);
        for (int t = 0; t < p.n_inj; ++t) {
            const int r = inj[t].row - (row0 + wm * WTM), c = inj[t].col - (col0 + wn * WTN);
            const uint32_t mask = inj[t].xor_mask;
            if (r < 0 || r >= WTM || c < 0 || c >= WTN) continue;
            if (inj[t].row >= p.M || inj[t].col >= p.N) continue;
            const int bi = r >> 5, rr = r & 31, bj = c >> 5;
            const int e_hit = (rr >> 3) * 4 + (rr & 3), half_hit = (rr >> 2) & 1;
            const bool mine = (lcol == (c & 31)) && (lhalf == half_hit);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (mine && i == bi && j == bj && e == e_hit) acc[i][j][e] ^= (int)mask;
        }
    }

    int32_t atom_old = 0;
    if (kCheck) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                uint32_t s = 0;
#pragma unroll
                for (int j = 0; j < TN; ++j) s += (uint32_t)acc[i][j][e];
#pragma unroll
                for (int off = 1; off < 32; off <<= 1) s += (uint32_t)__shfl_xor((int)s, off);
                if (lcol == 0) s_rs[wn * BM + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * lhalf + (e & 3)] = (int32_t)s;
            }
        // 16x16 accumulator: lane l, element e is row 4*(l/16) + e, column l%16; columns
        // 0..3 hold the four digit products.
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int d = lane & 15;
                uint32_t v = d < kLimbs ? ((uint32_t)cacc[c][e] << (8 * d)) : 0u;
                v += (uint32_t)__shfl_xor((int)v, 1);
                v += (uint32_t)__shfl_xor((int)v, 2);
                if (d == 0) s_ck[wm * WTM + (wn * CB + c) * 16 + 4 * (lane >> 4) + e] = (int32_t)v;
            }
        __syncthreads();
        for (int r = tid; r < BM; r += NT) {
            if (row0 + r < p.M) {
                uint32_t d = 0;
#pragma unroll
                for (int w = 0; w < WGN; ++w) d += (uint32_t)s_rs[w * BM + r];
                d -= (uint32_t)s_ck[r];
                if (tile_n == 0) d -= 128u * (uint32_t)(*p.total);  // sum_k 128*S_B[k], once per row
                // fetch-add WITH return: once the old value is back the add has been
                // performed at device scope, which is what the arrival counter relies on
                if (d != 0)
                    atom_old |= __hip_atomic_fetch_add(p.ws + kWsHeaderInts + row0 + r, (int)d, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }

    // store C_temp and/or its requantized form; padded rows and columns are dropped.  The
    // zero-point term of Eq. 1 uses the column sums stored with the weight.
    RequantCol rqc[TN];   // this lane's columns, fetched once ahead of the stores
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        rqc[j].sub = 0;
        rqc[j].mult = 0.0f;
        if (kWantQ) {
            const int col = col0 + wn * WTN + j * 32 + lcol;
            rqc[j] = requant_col(p.colsum[col], col < p.N ? col : 0, p.rq);
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = row0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * lhalf + (e & 3);
            if (row < p.M) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = col0 + wn * WTN + j * 32 + lcol;
                    if (col < p.N) {
                        if (kWantC) p.C[(int64_t)row * p.ldc + col] = acc[i][j][e];
                        if (kWantQ) p.Cq[(int64_t)row * p.ldcq + col] = requant_with(acc[i][j][e], rqc[j], p.rq.zC);
                    }
                }
            }
        }

    if (kCheck) {
        // The last workgroup to arrive turns the accumulated differences into flags and
        // puts the workspace back to zero.  No cache maintenance is involved: all data that
        // crosses workgroups moves through device-scope atomics, and every thread has its
        // fetch-add result back (the store of atom_old below waits for it) before the
        // barrier that precedes the arrival count.
        s_bs[tid] = atom_old;
        __syncthreads();
        if (tid == 0) {
            uint32_t unused = 0;
            s_ctl[0] = arrive_two_level(p.ws, 0u, gridDim.x, blockIdx.x, &unused);
            s_ctl[1] = 0;
        }
        __syncthreads();
        if (s_ctl[0]) {
            int cnt = 0;
            for (int r0 = 0; r0 < p.M; r0 += NT * 8) {
                // eight independent device-scope loads in flight per thread, then the stores
                int d[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = r0 + u * NT + tid;
                    d[u] = r < p.M ? __hip_atomic_load(p.ws + kWsHeaderInts + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = r0 + u * NT + tid;
                    if (r < p.M) {
                        if (d[u] != 0)
                            __hip_atomic_store(p.ws + kWsHeaderInts + r, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        p.row_flags[r] = d[u] != 0;
                        cnt += d[u] != 0;
                    }
                }
            }
            if (cnt) atomicAdd(&s_ctl[1], cnt);
            __syncthreads();
            if (tid == 0 && p.err_count) {
                if (!p.err_accumulate) *p.err_count = s_ctl[1];
                else if (s_ctl[1]) atomicAdd(p.err_count, s_ctl[1]);
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN>
hipError_t launch_cfg(bool check, bool want_c, bool want_q, const GemmParams& p, hipStream_t s) {
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(WGM * WGN * 64);
    const size_t lds = 2 * (BM + BN) * 64;
#define ABFT_LAUNCH(CK, OUT)                                                                              \
    do {                                                                                                  \
        auto kern = gemm_tile_kernel<BM, BN, WGM, WGN, CK, OUT>;                                          \
        static std::atomic<uint64_t> lds_allowed{0};                                                      \
        const hipError_t e_attr = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds, lds_allowed);\
        if (e_attr != hipSuccess) return e_attr;                                                          \
        kern<<<grid, block, lds, s>>>(p, tiles_n);                                                        \
        return hipGetLastError();                                                                         \
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

}  // namespace tile
}  // namespace abft
