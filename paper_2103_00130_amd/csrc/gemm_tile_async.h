// Checked u8 x s8 -> s32 GEMM for gfx950: LDS-tiled int8-MFMA kernel whose tiles are
// filled by direct global->LDS loads (the fast path: A and lda multiples of 16 bytes,
// K a multiple of 16).
//
// Algorithm 1 of arXiv 2103.00130 from the product line on: C_temp = A * [B | S_B] in ONE
// pass over A (Section IV-A-3, the checksum rides the level-3 product), then tSum per row,
// the comparison of Eq. 2b and errCount, then (optionally) the requantization of
// Section III-B, which never sees the checksum column (Section IV-B).
//
// Mapping to the hardware
//  * Stage = 128 k-values.  A rows are fetched as whole 128-byte lines (8 lanes x 16 B per
//    row) straight into LDS; each lane picks the 16-byte chunk  slot ^ ((row >> 1) & 7)  of
//    its row, so the 128-byte-pitch LDS image is XOR-swizzled and the MFMA fragment reads
//    (32 rows x 16 B) spread over all banks.  Packed B is already in fragment order and is
//    copied 1 KiB per wavefront instruction.  kStages stages are resident; their loads are
//    spread over the k-steps of the stages before them and one barrier per stage publishes
//    the next stage and releases the oldest.
//  * A is uint8, the matrix cores are signed x signed: fragments of A are XOR-ed with 0x80
//    (a - 128) after the LDS read and 128 * (column sum of the streamed B bytes) is added
//    back on the way to memory: exact modulo 2^32 for whatever B is in memory.
//  * The int32 checksum column S_B enters the same MFMA pipeline as four signed base-256
//    digit columns (a fifth B operand with 4 live columns); the tile columns of the grid
//    split its K range (tile column c takes a contiguous share of the stages).  Row sums are
//    formed while C is stored; each row's (row sum - checksum) share goes to the row's 64-bit
//    workspace word with one returned atomic that also counts arrivals, and the tile column
//    that arrives last writes the row's flag.
//  * With p.mod127 the same kernel follows Algorithm 1 to the letter: the fifth operand is
//    rowSum = S_B mod 127 (one live digit column) and the row sums are kept unwrapped and
//    reduced modulo 127 (Section IV-A-2).
#pragma once
#include <type_traits>

#include "../../include/abft_gemm.h"
#include "abft_internal.h"

namespace abft {
namespace atile {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kOutC = 1, kOutQ = 2;
constexpr int BK = 128;  // k-values per stage

// sum over the 32 lanes that share lane>>5: DPP adds inside rows of 16 lanes, then one
// v_permlane16_swap (rows 0<->1 and 2<->3 change places) for the last step; all VALU
__device__ inline uint32_t sum32(uint32_t s) {
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0x141, 0xF, 0xF, true);  // row_half_mirror
    s += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, 0x140, 0xF, 0xF, true);  // row_mirror
    const auto sw = __builtin_amdgcn_permlane16_swap(s, s, false, false);
    return sw[0] + sw[1];
}

// Sums over the 32 lanes that share lane>>5, for sixteen values per lane at once: a reduce-scatter.
// At each of four steps a lane keeps one half of the values it still holds, chosen by one bit of its
// lane number, and adds what its partner (the lane that differs in that bit) sends of the same half;
// a fifth step adds the two rows of sixteen lanes.  Lane l ends up with the complete sum of value
// number 8*l0 + 4*l1 + 2*l2 + l3 (l_k = bit k of l): 31 cross-lane additions instead of 16 x 5, in
// chains that do not depend on each other.
__device__ inline uint32_t sum32_of16(const uint32_t (&v)[16], int lane) {
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4, b3 = lane & 8;
    uint32_t w[8], x[4], y[2];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t keep = b0 ? v[8 + j] : v[j], send = b0 ? v[j] : v[8 + j];
        w[j] = keep + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0xB1, 0xF, 0xF, true);   // lane ^ 1
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t keep = b1 ? w[4 + j] : w[j], send = b1 ? w[j] : w[4 + j];
        x[j] = keep + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0x4E, 0xF, 0xF, true);   // lane ^ 2
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t keep = b2 ? x[2 + j] : x[j], send = b2 ? x[j] : x[2 + j];
        y[j] = keep + (uint32_t)__builtin_amdgcn_ds_swizzle((int)send, 0x101F);                     // lane ^ 4
    }
    const uint32_t keep = b3 ? y[1] : y[0], send = b3 ? y[0] : y[1];
    const uint32_t z = keep + (uint32_t)__builtin_amdgcn_ds_swizzle((int)send, 0x201F);             // lane ^ 8
    const auto sw = __builtin_amdgcn_permlane16_swap(z, z, false, false);                            // lane ^ 16
    return sw[0] + sw[1];
}

// v mod 127 in [0,126] for |v| < 2^59: 2^28 = (2^7)^4 is 1 modulo 127, so the two parts of
// v = hi * 2^28 + lo (floor split) may simply be added before the 32-bit remainder
__device__ inline int32_t floor_mod127(long long v) {
    const int32_t x = (int32_t)(v >> 28) + (int32_t)(v & 0x0FFFFFFF);
    const int32_t r = x % 127;
    return r < 0 ? r + 127 : r;
}

// kBlockSums: the cross-lane part of the row sums is done for the sixteen rows of a block together
// (sum32_of16) instead of row by row between the stores; the launcher says when.
// LDS bytes of one group of WGM x WGN wavefronts: the stage ring, the scratch of the epilogue, the staged
// checksum digits (kLimbStages stages of 512 bytes)
template <int BM, int BN, int WGN, int kStages, int WGK>
constexpr size_t group_lds_bytes() {
    return kStages * (size_t)(BM + BN) * BK + (4 * BN + WGN * BM + BM + 4) * sizeof(int32_t) + (32 / WGK) * 512;
}

// WGK > 1: K split inside the workgroup.  WGK groups of WGM x WGN wavefronts work on the same tile; group g
// takes the g-th run of stages with a stage ring of its own, so that a SIMD has WGK wavefronts to issue
// from (a tile of 64x64 keeps one wavefront per SIMD busy with about a hundred instructions per stage,
// and one wavefront issues at most one instruction every four cycles).  The groups pass the same
// barriers (same number of stages each, the launcher sees to it); at the end groups 1.. hand their
// accumulators to group 0 through LDS and leave, and group 0 runs the epilogue.
// kSplitK: K split across workgroups as well.  p.ksplit workgroups per tile take consecutive runs of stages; each
// stores its partial tile (accumulators and column sums) in the workspace and takes a ticket on the tile's counter,
// and the one that arrives last adds the others' partials to its own and runs the epilogue.  The checksum product
// of every run of stages is dealt out to the tile columns as before, so every workgroup contributes its share
// of it to the row words directly (the comparison of Eq. 2b is linear in the K slices) and only the last one
// contributes row sums.  For grids of 64x64 tiles that would leave most compute units idle.
template <int BM, int BN, int WGM, int WGN, int kStages, bool kCheck, int kOut, bool kBlockSums, int WGK, bool kSplitK = false>
__global__ __launch_bounds__(WGM* WGN* WGK * 64) void gemm_tile_async_kernel(const GemmParams p, const int tiles_m,
                                                                             const int tiles_n) {
    constexpr int NW = WGM * WGN, NT = NW * 64;    // wavefronts and threads of one group
    constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 blocks per wave
    constexpr int A_STAGE = BM * BK, B_STAGE = BN * BK;
    constexpr int S = kStages;                     // stages resident in LDS
    static_assert(S >= 2, "at least a double buffer");
    constexpr int A_LD = (BM / 8) / NW;            // async A loads per wave per stage (8 rows each)
    constexpr int B_LD = (BN / 8) / NW;            // async B loads per wave per stage (1 KiB each)
    constexpr int CB = (WTM / 16) / WGN;           // 16-row checksum blocks per wave
    constexpr bool kWantC = (kOut & kOutC) != 0, kWantQ = (kOut & kOutQ) != 0;
    static_assert(A_LD >= 1 && B_LD >= 1 && CB >= 1 && (WTM / 16) % WGN == 0, "tile too small for the workgroup");
    static_assert(BN >= 64 && NT <= 4 * BN, "epilogue scratch layout");

    // LDS of a group: [S][A_STAGE] then [S][B_STAGE], then the scratch of the epilogue, then the digits
    extern __shared__ __align__(1024) uint8_t smem_all[];
    constexpr size_t GROUP_LDS = (group_lds_bytes<BM, BN, WGN, kStages, WGK>() + 1023) / 1024 * 1024;
    const int grp = WGK > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x / NT) : 0;
    uint8_t* const smem = smem_all + grp * GROUP_LDS;
    const uint32_t lds_base = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) uint8_t*)smem);

    const int tid = (int)threadIdx.x - grp * NT, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    // Workgroups go round-robin over the 8 XCDs; give every XCD a compact block of tiles
    // (consecutive ids inside an XCD walk down a strip of 4 tile rows) so that its L2 sees
    // few distinct A and B panels.
    int tile_m, tile_n;
    {
        const int n_tiles = tiles_m * tiles_n;
        int t = kSplitK ? (int)blockIdx.x % n_tiles : (int)blockIdx.x;   // (split-K: slice z = blockIdx.x / n_tiles)
        if (!kSplitK && n_tiles % 8 == 0) t = (blockIdx.x & 7) * (n_tiles >> 3) + (blockIdx.x >> 3);
        const int strip_h = tiles_m >= 4 ? 4 : tiles_m;
        const int per_strip = strip_h * tiles_n;
        const int strip = t / per_strip, r = t - strip * per_strip;
        const int h = min(strip_h, tiles_m - strip * strip_h);  // last strip may be shorter
        tile_n = r / h;
        tile_m = strip * strip_h + r - tile_n * h;
    }
    const int row0 = tile_m * BM, col0 = tile_n * BN;
    const int Z = kSplitK ? p.ksplit : 1;                                       // K slices across workgroups
    const int z = kSplitK ? (int)blockIdx.x / (tiles_m * tiles_n) : 0;
    const int NS_all = p.KB2;            // stages of 128 k-values
    const int NS = NS_all / (WGK * Z);   // ... of this group (the launcher splits only what divides)
    const int s_base = (z * WGK + grp) * NS;  // its first stage

    // ---- direct global->LDS loads ---------------------------------------------------
    // One instruction moves 16 bytes per lane to LDS address m0 + lane*16.  They are issued
    // through inline asm so that the compiler keeps treating the LDS reads of the resident
    // stage as independent of them; completion is awaited explicitly (vmcnt) before the
    // barrier that publishes a stage.
    // Addresses: a uniform base in scalar registers (advanced by the stage) plus a 32-bit
    // per-lane offset that never changes, so that a load costs no vector address arithmetic.
    auto dma = [](uint32_t lds_addr, uint32_t voff, const void* sbase, auto off_c) __attribute__((always_inline)) {
        constexpr int OFF = decltype(off_c)::value;  // added to the global AND to the LDS address
        // one wait state between the write of m0 and the instruction that reads it
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
                     ::"s"(lds_addr), "v"(voff), "s"(sbase), "n"(OFF) : "m0", "memory");
    };
    // A: instruction i of this wave covers rows (wave*A_LD + i)*8 .. +8 of the tile; lane l
    // takes row l>>3 of those and the 16-byte chunk (l&7) ^ ((row>>1)&7) of the stage.  In the
    // last stage a chunk at or past K is re-read from the last whole chunk (it meets zero rows
    // of B), hence the second set of offsets.
    uint32_t a_voff[A_LD], a_voff_last[A_LD], a_lds[A_LD];
    {
        const int c16_max = p.K - 16 - (NS_all - 1) * BK;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int r = (wave * A_LD + i) * 8 + (lane >> 3);
            const int c16 = ((lane & 7) ^ ((r >> 1) & 7)) * 16;
            const uint32_t rowoff = (uint32_t)min(row0 + r, p.M - 1) * (uint32_t)p.lda;
            a_voff[i] = rowoff + (uint32_t)c16;
            a_voff_last[i] = rowoff + (uint32_t)((grp == WGK - 1 && z == Z - 1) ? min(c16, c16_max) : c16);  // only the last group meets K's end
            a_lds[i] = lds_base + (wave * A_LD + i) * 1024;
        }
    }
    constexpr int TILES_PER_NT = kTileN / BN;
    constexpr int64_t B_KB_STRIDE = (int64_t)kUnitsPerTile * kUnitBytes;
    constexpr int B_CHUNKS_PER_KB = BN / 16;  // 1 KiB chunks of this tile per k-block of 64
    static_assert(B_CHUNKS_PER_KB % B_LD == 0, "the chunks of one wave lie in one k-block");
    // B: this wave copies B_LD consecutive 1 KiB chunks of the stage; packed B and its LDS image
    // have the same order, so one base pair serves four loads through the instruction offset.
    const int8_t* b_wave;
    uint32_t b_lds;
    const uint32_t b_voff = lane * 16;
    {
        const int bc0 = wave * B_LD, kbl = bc0 / B_CHUNKS_PER_KB, cc0 = bc0 % B_CHUNKS_PER_KB;
        b_wave = p.packed + packed_unit_offset(tile_n / TILES_PER_NT, 0, (tile_n % TILES_PER_NT) * (BN / 32), p.KB2 * 2) +
                 (int64_t)kbl * B_KB_STRIDE + cc0 * 1024 + (int64_t)s_base * (2 * B_KB_STRIDE);
        b_lds = lds_base + S * A_STAGE + kbl * (BN * 64) + cc0 * 1024;
    }

    // load n of stage s into buffer buf: n < A_LD is an A load (8 rows x 128 B), the rest are
    // B loads (1 KiB of packed B each).
    constexpr int N_LD = A_LD + B_LD;
    auto issue_load = [&](int s, int buf, int n) __attribute__((always_inline)) {
        if (n < A_LD) {
            const uint32_t voff = (s == NS - 1) ? a_voff_last[n] : a_voff[n];
            dma(a_lds[n] + buf * A_STAGE, voff, p.A + (int64_t)(s_base + s) * BK, std::integral_constant<int, 0>{});
        } else {
            const int j = n - A_LD, g = j >> 2;
            const int8_t* const base = b_wave + (int64_t)s * (2 * B_KB_STRIDE) + g * 4096;
            const uint32_t l = b_lds + buf * B_STAGE + g * 4096;
            switch (j & 3) {
                case 0: dma(l, b_voff, base, std::integral_constant<int, 0>{}); break;
                case 1: dma(l, b_voff, base, std::integral_constant<int, 1024>{}); break;
                case 2: dma(l, b_voff, base, std::integral_constant<int, 2048>{}); break;
                default: dma(l, b_voff, base, std::integral_constant<int, 3072>{}); break;
            }
        }
    };

    // ---- fragment reads -----------------------------------------------------------
    // A fragment (block i, k-step j): lane l holds row wm*WTM + i*32 + (l&31), chunk 2j + (l>>5)
    const int a_swz = (lane >> 1) & 7;
    int a_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) a_off[j] = (wm * WTM + (lane & 31)) * BK + (((2 * j + (lane >> 5)) ^ a_swz) << 4);
    const int b_off = S * A_STAGE + wn * TN * 2048 + lane * 16;

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
    // column sums of the B bytes streamed (every wave keeps them for its own columns)
    uint32_t bsum[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bsum[j] = 0;

    // Small wave tiles (at most four MFMAs per k-step) read their fragments two k-steps ahead: one
    // k-step of such a tile is shorter than the latency of an LDS read, so with one k-step of
    // lookahead every k-step would end in a wait for its successor's operands.  Four fragment sets,
    // one per k-step of a stage.
    constexpr bool kAhead2 = TM * TN <= 4;
    constexpr int NSETS = kAhead2 ? 4 : 2;
    v4i fa[NSETS][TM], fb[NSETS][TN];
    auto read_frags = [&](int buf, int j, int f) __attribute__((always_inline)) {
        const uint8_t* sA = smem + buf * A_STAGE;
        const uint8_t* sB = smem + buf * B_STAGE;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[f][i] = *reinterpret_cast<const v4i*>(sA + a_off[j] + i * 32 * BK);
#pragma unroll
        for (int t = 0; t < TN; ++t)
            fb[f][t] = *reinterpret_cast<const v4i*>(sB + (j >> 1) * (BN * 64) + b_off + t * 2048 + (j & 1) * 1024);
    };
    // Checksum digits as the B operand of a 16x16x64 MFMA (one per k-block of the stage):
    // lane l holds digit column l&15 (zero beyond 3) and k-group l>>4.  The matching A operand
    // is row (l&15) of a 16-row block, chunk 4*kbl + (l>>4) of the stage.
    v4i limb[2];
    limb[0] = limb[1] = v4i{0, 0, 0, 0};
    // This tile column's contiguous share [ck_lo, ck_hi) of the checksum product's K range.  Its
    // digits (512 bytes per stage) are staged in LDS, kLimbStages stages at a time: the first lot
    // behind the loads of the first stages, a further lot (shares longer than that: K beyond
    // 4096 per tile column) between two runs of stages.  The stages that use them read LDS, so
    // that the loop holds no global load the compiler knows of: it would put a wait for *all*
    // vector-memory traffic, the direct-to-LDS loads of the next stage included, in front of the
    // digit MFMAs.
    constexpr int kLimbStages = 32 / WGK;
    // (stage numbers of this group: every group's run of stages is dealt out to the tile columns in the same way, so
    // that the groups of a K-split workgroup carry the same number of checked stages between their common barriers)
    const int ck_lo = kCheck ? share_begin(tile_n, p.share_q, p.share_r) : 0;
    const int ck_hi = kCheck ? share_begin(tile_n + 1, p.share_q, p.share_r) : 0;
    uint8_t* const s_limb = smem + S * (A_STAGE + B_STAGE) + (4 * BN + WGN * BM + BM + 4) * sizeof(int32_t);
    // sum_k S_B[k], which the first tile column needs at the very end (the u8 -> s8 shift of A moves every
    // checksum product by 128 times it): fetched now, so that the epilogue does not wait for memory
    int32_t total_sb = (kCheck && tile_n == 0 && z == 0) ? *p.total : 0;
    int limb_base = ck_lo;  // stage whose digits sit at the start of s_limb
    // (copied by the same direct global->LDS loads as the stages, 1 KiB per instruction: no trip through
    // registers, and no wait that the compiler would place - it does not see the direct loads and would
    // wait for every one of them.  A lot that ends in half an instruction re-reads its last chunk into
    // LDS words behind the lot, which nobody reads.)
    const uint32_t lds_limb = lds_base + (uint32_t)(S * (A_STAGE + B_STAGE) + (4 * BN + WGN * BM + BM + 4) * sizeof(int32_t));
    auto stage_limbs = [&](int s0) __attribute__((always_inline)) {
        const int n = min(ck_hi - s0, kLimbStages);
        const int8_t* const src = p.limbs + (int64_t)(s_base + s0) * 512;
        for (int i = wave; i * 2 < n; i += NW)
            dma(lds_limb + i * 1024, (uint32_t)min(i * 1024 + lane * 16, n * 512 - 16), src, std::integral_constant<int, 0>{});
        limb_base = s0;
    };
    auto load_limbs = [&](int s) __attribute__((always_inline)) {
        // this lane's digit inside a k-block.  Lanes of columns 4..15 read the last digit again: what they
        // feed the MFMA lands in result columns that nobody reads, and an unconditional read costs no
        // branch and no wait of its own.
        const int q = ((lane >> 4) * kLimbs + min(lane & 15, kLimbs - 1)) << 4;
#pragma unroll
        for (int kbl = 0; kbl < 2; ++kbl) limb[kbl] = *reinterpret_cast<const v4i*>(s_limb + ((s - limb_base) * 2 + kbl) * 256 + q);
    };
    // The digit MFMA with its accumulator in ordinary vector registers.  All 256 accumulation
    // registers hold the tile; left to the compiler, the digit accumulators would be swapped into
    // them and out again around every digit MFMA (it gives every MFMA of a function the same
    // register class for its result).  The instruction takes either class, so it is written out
    // here; the two wait states that a vector write needs before a matrix instruction reads the
    // register (the XOR on the operand) are part of the string, since no hazard pass sees inside it.
    auto mfma_digits = [](v4i& c, v4i a, v4i b) __attribute__((always_inline)) {
        asm volatile("s_nop 1\n\tv_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
    };
    int ck_off[2];
#pragma unroll
    for (int kbl = 0; kbl < 2; ++kbl)
        ck_off[kbl] = (wm * WTM + wn * CB * 16 + (lane & 15)) * BK + (((4 * kbl + (lane >> 4)) ^ a_swz) << 4);
    auto wait_lds = []() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xC07F); };
    auto wait_vmem = []() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0x0F70); };
    // at most n LDS operations still in flight (they complete in order)
    auto wait_lds_but = [](auto n_c) __attribute__((always_inline)) {
        constexpr int n = decltype(n_c)::value;
        static_assert(n >= 0 && n < 16, "lgkmcnt is a 4-bit field");
        __builtin_amdgcn_s_waitcnt(0xC07F | (n << 8));
    };
    // at most n vector-memory operations still in flight (they complete in order)
    auto wait_vmem_but = [](auto n_c) __attribute__((always_inline)) {
        constexpr int n = decltype(n_c)::value;
        static_assert(n >= 0 && n < 64, "vmcnt is a 6-bit field");
        __builtin_amdgcn_s_waitcnt(((n >> 4) << 14) | (n & 15) | 0x0F70);
    };

    // One k-step of 32: TM x TN MFMAs on fragment set f while fragment set fr is read for
    // k-step jn of buffer rbuf and loads [ld_lo, ld_hi) of stage ld_s go out to buffer ld_buf.
    // The k-step is cut into regions of two MFMAs that the instruction scheduler may not move
    // anything across; each region carries its share of the other work, so that every LDS
    // read, vector-memory instruction and VALU instruction issues in the shadow of an MFMA:
    //  * the LDS reads of the next fragments go into the first half of the regions, so that
    //    they have returned when the k-step ends;
    //  * a - 128 as int8 (XOR 0x80 on data already in registers) for the next row of blocks is
    //    computed one row ahead of its first MFMA;
    //  * when SUM_B, the B bytes of this k-step are added into the column sums: XOR 0x80 turns
    //    int8 into a biased uint8 whose four bytes v_sad_u8 sums against zero (the bias, 128
    //    per byte, is taken off in the epilogue);
    //  * the direct-to-LDS loads are spread evenly instead of arriving in a burst.
    auto phase = [&](int f, int fr, int rbuf, int jn, auto sum_b_c, int ld_s, int ld_buf, int ld_lo, int ld_hi)
                     __attribute__((always_inline)) {
        constexpr bool SUM_B = decltype(sum_b_c)::value;
        constexpr int Q = TM * TN, NR = Q / 2, R = TM + TN, RR = NR >= 2 ? NR / 2 : 1, D = 4 * TN;
        static_assert(TN % 2 == 0, "regions pair the MFMAs of one row of blocks");
        const uint8_t* const sA = smem + rbuf * A_STAGE + a_off[jn];
        const uint8_t* const sB = smem + rbuf * B_STAGE + (jn >> 1) * (BN * 64) + b_off + (jn & 1) * 1024;
        v4i a_cur = fa[f][0] ^ (int)0x80808080, a_nxt = a_cur;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = (2 * r) / TN, t0 = (2 * r) % TN;
            if (t0 == 0 && i + 1 < TM) a_nxt = fa[f][i + 1] ^ (int)0x80808080;
            acc[i][t0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a_cur, fb[f][t0], acc[i][t0], 0, 0, 0);
            acc[i][t0 + 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a_cur, fb[f][t0 + 1], acc[i][t0 + 1], 0, 0, 0);
            if (r < RR) {
#pragma unroll
                for (int x = R * r / RR; x < R * (r + 1) / RR; ++x) {
                    if (x < TM) fa[fr][x] = *reinterpret_cast<const v4i*>(sA + x * 32 * BK);
                    else fb[fr][x - TM] = *reinterpret_cast<const v4i*>(sB + (x - TM) * 2048);
                }
            }
            if (SUM_B) {
#pragma unroll
                for (int d = D * r / NR; d < D * (r + 1) / NR; ++d)
                    bsum[d >> 2] = __builtin_amdgcn_sad_u8((uint32_t)fb[f][d >> 2][d & 3] ^ 0x80808080u, 0u, bsum[d >> 2]);
            }
#pragma unroll
            for (int n = ld_lo + (ld_hi - ld_lo) * r / NR; n < ld_lo + (ld_hi - ld_lo) * (r + 1) / NR; ++n)
                issue_load(ld_s, ld_buf, n);
            if (t0 + 2 >= TN) a_cur = a_nxt;
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The same k-step for small wave tiles (at most four MFMAs): too short to be cut into regions.
    // Reads first, then the MFMAs with the vector work behind them.
    auto phase_small = [&](int f, int fr, int rbuf, int jn, auto sum_b_c, int ld_s, int ld_buf, int ld_lo, int ld_hi)
                           __attribute__((always_inline)) {
        constexpr bool SUM_B = decltype(sum_b_c)::value;
        const uint8_t* const sA = smem + rbuf * A_STAGE + a_off[jn];
        const uint8_t* const sB = smem + rbuf * B_STAGE + (jn >> 1) * (BN * 64) + b_off + (jn & 1) * 1024;
#pragma unroll
        for (int x = 0; x < TM; ++x) fa[fr][x] = *reinterpret_cast<const v4i*>(sA + x * 32 * BK);
#pragma unroll
        for (int x = 0; x < TN; ++x) fb[fr][x] = *reinterpret_cast<const v4i*>(sB + x * 2048);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const v4i a = fa[f][i] ^ (int)0x80808080;
#pragma unroll
            for (int t = 0; t < TN; ++t) acc[i][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, fb[f][t], acc[i][t], 0, 0, 0);
        }
        if (SUM_B) {
#pragma unroll
            for (int d = 0; d < 4 * TN; ++d)  // signed byte sums, one instruction per word (no bias to take off later)
                bsum[d >> 2] = (uint32_t)__builtin_amdgcn_sdot4(fb[f][d >> 2][d & 3], 0x01010101, (int)bsum[d >> 2], false);
        }
#pragma unroll
        for (int n = ld_lo; n < ld_hi; ++n) issue_load(ld_s, ld_buf, n);
        __builtin_amdgcn_sched_barrier(0);
    };

    // Load schedule.
    // Double buffer (S = 2): 3/8 of the loads of stage s+1 go out during the last k-step of
    // stage s-1, 3/8 during the first and 2/8 during the second k-step of stage s (measured best
    // among the even spreads; issuing any in the third k-step leaves them too little time to
    // land before the barrier that follows it).
    // Ring (S > 2, the small tiles, whose k-steps are too short to cover the latency of a load
    // with one stage of lookahead): the slot of stage s is released by the barrier that follows
    // its third k-step and is refilled with stage s+S, a quarter per k-step from the fourth
    // k-step of stage s on; a stage therefore has S-1 stages of time to land, and at each
    // barrier only what is older than the (S-2)*N_LD most recent loads is awaited.
    constexpr int LD_C0 = S == 2 ? N_LD * 3 / 8 : N_LD / 4, LD_C1 = S == 2 ? N_LD * 6 / 8 : N_LD / 2,
                  LD_C2 = S == 2 ? N_LD : N_LD * 3 / 4;
    using pending_c = std::integral_constant<int, (S - 2) * N_LD>;
    // Two k-steps of lookahead (kAhead2): all S slots are filled before the loop; in stage s the first two
    // k-steps read the last two fragment sets of the stage, a barrier then publishes stage s+1 and
    // releases the slot of stage s (everything read from it is in registers), and the last two
    // k-steps read the first two fragment sets of stage s+1 while the loads of stage s+S go out, one
    // half per k-step, to the slot just released.
    using frag_reads_c = std::integral_constant<int, TM + TN>;  // LDS reads of one k-step
    // (the digits of this tile column's share go out first: whatever wait publishes the first stage then
    // covers them as well, and their round trip to memory runs beside that of the stages)
    if constexpr (kAhead2) {
        if (kCheck && ck_hi > ck_lo) stage_limbs(ck_lo);
#pragma unroll
        for (int st = 0; st < S; ++st)
#pragma unroll
            for (int n = 0; n < N_LD; ++n) issue_load(min(st, NS - 1), st, n);
        wait_vmem_but(std::integral_constant<int, (S - 1) * N_LD>{});
        __syncthreads();
        read_frags(0, 0, 0);
        read_frags(0, 1, 1);
        wait_lds();
        __builtin_amdgcn_sched_barrier(0);
    } else {
        if (kCheck && ck_hi > ck_lo) stage_limbs(ck_lo);
#pragma unroll
        for (int st = 0; st < S - 1; ++st)
#pragma unroll
            for (int n = 0; n < N_LD; ++n) issue_load(min(st, NS - 1), st, n);
        wait_vmem_but(pending_c{});
        __syncthreads();
        // first share of the stage after those
#pragma unroll
        for (int n = 0; n < LD_C0; ++n) issue_load(min(S - 1, NS - 1), S - 1, n);
        read_frags(0, 0, 0);
        wait_lds();
        __builtin_amdgcn_sched_barrier(0);
    }

    asm volatile("" : "+s"(total_sb));  // (the value is in its register from here on)
#ifdef ABFT_CLOCK_TRACE
    // Diagnostic build only: the first thread of every workgroup samples the shader-clock cycle counter and the
    // constant 100 MHz wall counter before the K loop, after it and at the end of the kernel (6 words per
    // workgroup): cycles over wall time is the clock the chip sustained in each phase.
    unsigned long long trace_c0 = clock64(), trace_r0 = wall_clock64();
#endif
    int cur = 0;
    // A run of stages [s_begin, s_end) with or without the checksum-digit MFMAs (separate loops
    // keep every loop body one straight block).  PH says on which k-steps this wave adds the B
    // bytes it holds into the column sums: the waves that share a column range (same wn) take
    // alternate k-steps (0: even, 1: odd), a lone wave takes all (2).
    // Load schedule: see the cut points above; the loads of stage s+1 are awaited at the end of
    // the third k-step of stage s, where the single barrier of the stage sits.  A stage index
    // past the end re-reads the last stage into a dead buffer.
    auto run = [&](int s_begin, int s_end, auto chk_c, auto ph_c) __attribute__((always_inline)) {
        constexpr bool CHK = decltype(chk_c)::value;
        constexpr int PH = decltype(ph_c)::value;
        using even_c = std::integral_constant<bool, PH != 1>;
        using odd_c = std::integral_constant<bool, PH != 0>;
        // checksum-digit columns for this wave's share of the rows (16-row blocks wn*CB ..) over both
        // k-blocks of the stage in slot `buf`; the A operands are re-read from the resident stage
        auto digit_block = [&](int buf) __attribute__((always_inline)) {
            const uint8_t* sA = smem + buf * A_STAGE;
#pragma unroll
            for (int kbl = 0; kbl < 2; ++kbl) {
                v4i av[CB];
#pragma unroll
                for (int c = 0; c < CB; ++c) av[c] = *reinterpret_cast<const v4i*>(sA + ck_off[kbl] + c * 16 * BK);
#pragma unroll
                for (int c = 0; c < CB; ++c) mfma_digits(cacc[c], av[c] ^ (int)0x80808080, limb[kbl]);
            }
            // the digit accumulators are next read by vector instructions (epilogue) or by the digit
            // MFMAs of a later stage; cover the longest write-to-read distance of a 4-pass MFMA once
            asm volatile("s_nop 7\n\ts_nop 7");
        };
        // The same in two halves for the small wave tiles, whose stage is short enough for the latency
        // of these reads to show: the reads go out behind the last fragment reads of the stage, the
        // digit MFMAs follow the wait that those need anyway.
        v4i dig_a[2][CB];
        auto digit_reads = [&](int buf) __attribute__((always_inline)) {
            const uint8_t* sA = smem + buf * A_STAGE;
#pragma unroll
            for (int kbl = 0; kbl < 2; ++kbl)
#pragma unroll
                for (int c = 0; c < CB; ++c) dig_a[kbl][c] = *reinterpret_cast<const v4i*>(sA + ck_off[kbl] + c * 16 * BK);
        };
        auto digit_mfmas = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int kbl = 0; kbl < 2; ++kbl)
#pragma unroll
                for (int c = 0; c < CB; ++c) mfma_digits(cacc[c], dig_a[kbl][c] ^ (int)0x80808080, limb[kbl]);
            // (the digit accumulators are next touched a whole stage later, or after the wait states that
            // follow this run of stages)
        };
        if constexpr (kAhead2) {
            for (int s = s_begin; s < s_end; ++s) {
                const int nxt = cur + 1 == S ? 0 : cur + 1;
                const int s_new = min(s + S, NS - 1);  // refills the slot of this stage once it is released
                // the digit operands of this stage (it is resident) are read ahead of the fragments of its
                // first k-step and are there, reads completing in order, when the wait behind that k-step ends:
                // nothing of the digit work waits for LDS on its own
                if (CHK) {
                    load_limbs(s);
                    digit_reads(cur);
                }
                phase_small(0, 2, cur, 2, even_c{}, 0, 0, 0, 0);
                wait_lds_but(frag_reads_c{});
                __builtin_amdgcn_sched_barrier(0);
                if (CHK) digit_mfmas();
                phase_small(1, 3, cur, 3, odd_c{}, 0, 0, 0, 0);
                wait_lds();  // every fragment of this stage is in registers
                __builtin_amdgcn_sched_barrier(0);
                wait_vmem_but(pending_c{});
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                phase_small(2, 0, nxt, 0, even_c{}, s_new, cur, 0, N_LD / 2);
                wait_lds_but(frag_reads_c{});
                __builtin_amdgcn_sched_barrier(0);
                phase_small(3, 1, nxt, 1, odd_c{}, s_new, cur, N_LD / 2, N_LD);
                wait_lds_but(frag_reads_c{});
                __builtin_amdgcn_sched_barrier(0);
                cur = nxt;
            }
            // the last digit MFMAs of the run: cover the longest write-to-read distance once, whatever follows
            if (CHK) asm volatile("s_nop 7\n\ts_nop 7");
        } else {
            for (int s = s_begin; s < s_end; ++s) {
                // stage whose loads go out now, the slot they go to, and the slot of the next stage
                const int s1 = min(s + S - 1, NS - 1), s2 = min(s + S, NS - 1);
                const int nxt = cur + 1 == S ? 0 : cur + 1, tgt = cur == 0 ? S - 1 : cur - 1;
                // the digit operands of this stage are needed three quarters of a stage from now
                if (CHK) load_limbs(s);
                phase(0, 1, cur, 1, even_c{}, s1, tgt, LD_C0, LD_C1);
                wait_lds();
                __builtin_amdgcn_sched_barrier(0);
                phase(1, 0, cur, 2, odd_c{}, s1, tgt, LD_C1, LD_C2);
                wait_lds();
                __builtin_amdgcn_sched_barrier(0);
                phase(0, 1, cur, 3, even_c{}, s1, tgt, LD_C2, N_LD);
                wait_lds();
                __builtin_amdgcn_sched_barrier(0);
                if (CHK) digit_block(cur);
                // publish the next stage: this wave's loads of it have landed, and after the
                // barrier nobody reads the current stage any more
                wait_vmem_but(pending_c{});
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                phase(1, 0, nxt, 0, odd_c{}, s2, cur, 0, LD_C0);
                wait_lds();
                __builtin_amdgcn_sched_barrier(0);
                cur = nxt;
            }
        }
    };
    auto run_all = [&](auto ph_c) __attribute__((always_inline)) {
        if (kCheck) {
            run(0, ck_lo, std::false_type{}, ph_c);
            for (int c0 = ck_lo; c0 < ck_hi; c0 += kLimbStages) {
                if (c0 > ck_lo) {
                    // every wave has left the stages that read the previous lot (their digits were in
                    // registers before the barrier that ended the last of them)
                    stage_limbs(c0);
                    wait_vmem();
                    __syncthreads();
                }
                run(c0, min(c0 + kLimbStages, ck_hi), std::true_type{}, ph_c);
            }
            run(ck_hi, NS, std::false_type{}, ph_c);
        } else {
            run(0, NS, std::false_type{}, ph_c);
        }
    };
    if (WGM == 1) run_all(std::integral_constant<int, 2>{});
    else if ((wm & 1) == 0) run_all(std::integral_constant<int, 0>{});
    else run_all(std::integral_constant<int, 1>{});
    // (the last stage re-issued loads into a dead buffer; the epilogue keeps its scratch outside
    // the stage buffers, so nobody waits for them before the very end of the kernel)

#ifdef ABFT_CLOCK_TRACE
    if (p.clock_trace && threadIdx.x == 0) {
        unsigned long long* const o = p.clock_trace + (size_t)blockIdx.x * 6;
        o[0] = trace_c0;
        o[1] = trace_r0;
        o[2] = clock64();
        o[3] = wall_clock64();
    }
#endif
    // ------------------------- K split: the groups' results come together -------------------------
    if constexpr (WGK > 1) {
        static_assert(TM * TN <= 4, "the K split is for small wave tiles");
        constexpr int kVals = 16 * TM * TN + TN + 4 * CB;  // accumulators, column sums, digit accumulators per lane
        static_assert((size_t)kVals * NT * sizeof(int32_t) <= GROUP_LDS, "a group's values fit its own LDS");
        // every direct-to-LDS load of every group has landed and every wavefront has left the loop: the
        // LDS of groups 1.. is free (that of group 0 holds the scratch its epilogue is about to use)
        wait_vmem();
        __syncthreads();
        int32_t* const xch = reinterpret_cast<int32_t*>(smem_all + GROUP_LDS);
        if (grp > 0) {
            int32_t* const mine = xch + (size_t)(grp - 1) * kVals * NT + tid;
            int k = 0;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) mine[(k++) * NT] = acc[i][t][e];
#pragma unroll
            for (int t = 0; t < TN; ++t) mine[(k++) * NT] = (int32_t)bsum[t];
#pragma unroll
            for (int c = 0; c < CB; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e) mine[(k++) * NT] = cacc[c][e];
        }
        __syncthreads();
        if (grp > 0) return;  // (nothing of this group is in flight: its loads were awaited above)
#pragma unroll
        for (int g = 1; g < WGK; ++g) {
            const int32_t* const theirs = xch + (size_t)(g - 1) * kVals * NT + tid;
            int k = 0;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][t][e] += theirs[(k++) * NT];
#pragma unroll
            for (int t = 0; t < TN; ++t) bsum[t] += (uint32_t)theirs[(k++) * NT];
#pragma unroll
            for (int c = 0; c < CB; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e) cacc[c][e] += theirs[(k++) * NT];
        }
    }

    // ------------------------- K split across workgroups: partial tiles meet in the last arrival -------------------------
    bool last = true;   // this workgroup holds the complete tile (always, without a split)
    if constexpr (kSplitK) {
        static_assert(WGK == 1 && TM * TN == 1 && NT == 256, "split-K is built for the 64x64 tile of four 32x32 wavefronts");
        __shared__ int s_ticket;
        constexpr int kVals = 16 * TM * TN + TN;
        static_assert(kVals * NT == kSplitKPartInts, "layout of a partial tile");
        const int tile = tile_m * tiles_n + tile_n;
        int32_t* const mine = p.ws_part + ((size_t)tile * Z + z) * kSplitKPartInts + tid;
        {
            // device-scope stores (they pass through the L2, which is not coherent with the other seven): once this
            // wavefront's stores are acknowledged and the barrier is passed, the whole partial tile is in memory
            int k = 0;
#pragma unroll
            for (int e = 0; e < 16; ++e) __hip_atomic_store(mine + (k++) * NT, acc[0][0][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(mine + (k++) * NT, (int32_t)bsum[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        wait_vmem();   // (also the direct-to-LDS loads still in flight)
        __syncthreads();
        if (tid == 0) s_ticket = __hip_atomic_fetch_add(p.ws_tickets + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        last = s_ticket == Z - 1;
        if (last) {
            if (tid == 0) __hip_atomic_store(p.ws_tickets + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // the other slices' partial tiles, four at a time so that their loads are in flight together (a slice
            // number past the last one, or this workgroup's own, re-reads a valid partial and adds nothing)
            for (int z0 = 0; z0 < Z; z0 += 4) {
                int32_t v[4][kVals];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int32_t* const theirs = p.ws_part + ((size_t)tile * Z + min(z0 + j, Z - 1)) * kSplitKPartInts + tid;
#pragma unroll
                    for (int k = 0; k < kVals; ++k) v[j][k] = __hip_atomic_load(theirs + k * NT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int32_t use = (z0 + j < Z && z0 + j != z) ? -1 : 0;   // all ones or zero
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[0][0][e] += v[j][e] & use;
                    bsum[0] += (uint32_t)(v[j][16] & use);
                }
            }
        } else if (!kCheck) {
            return;   // (nothing in flight: awaited above)
        }
    }

    // ---------------------------------- epilogue ----------------------------------
    // accumulator layout of the 32x32 MFMA: lane l, element e of block (i, t) is
    // row 8*(e/4) + 4*(l/32) + e%4, column l%32 of that block.
    const int lcol = lane & 31, lhalf = lane >> 5;
    // LDS scratch behind the stage buffers: [4][BN] column sums, [WGN][BM] row-sum parts,
    // [BM] checksum parts, 4 control words
    int32_t* const s_bs = reinterpret_cast<int32_t*>(smem + S * (A_STAGE + B_STAGE));
    int32_t* const s_rs = s_bs + 4 * BN;
    int32_t* const s_ck = s_rs + WGN * BM;
    const bool mod127 = kCheck && p.mod127 != 0;
    // (split-K: only the workgroup that holds the complete tile stores it and forms its row sums)
    if (last) {
    // column sums of the streamed B: lane halves hold the two k-groups, waves wm = 0 and 1 (or a
    // lone wave) hold alternate k-steps; every byte carried a bias of 128
    constexpr int SUM_WAVES = WGM == 1 ? 1 : 2;
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const auto halves = __builtin_amdgcn_permlane32_swap(bsum[t], bsum[t], false, false);  // {own, lane ^ 32} in either order
        bsum[t] = halves[0] + halves[1];
        if (wm < SUM_WAVES && lhalf == 0) s_bs[wm * BN + wn * WTN + t * 32 + lcol] = (int32_t)bsum[t];
    }
    __syncthreads();
    int32_t cs[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        uint32_t v = (uint32_t)s_bs[wn * WTN + t * 32 + lcol];
        if (SUM_WAVES == 2) v += (uint32_t)s_bs[BN + wn * WTN + t * 32 + lcol];
        // (the k-steps of small wave tiles sum signed bytes directly, the others carry a bias of 128 per byte)
        cs[t] = 128 * (int32_t)(kAhead2 ? v : v - 128u * (uint32_t)(NS_all * BK));
    }
    // C_temp = accumulator + cs (undoing the a - 128 shift); the sum is formed on the way to
    // memory, the accumulators stay as they are
    // ---- stores, with the row sums of Eq. 2b formed on the way.  One running row pointer per
    // lane; it is laundered through an empty asm so that the 64 row addresses are produced one
    // after the other instead of all being kept in registers.  The stores are limited by how
    // fast memory takes them (several microseconds per tile), so the vector arithmetic placed
    // between them - the add-back, the row sums and their cross-lane reduction - costs nothing.
    int32_t cs_lane = 0;  // this lane's share of the add-back in a row sum
    long long cs_lane64 = 0;
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        cs_lane += cs[t];
        cs_lane64 += cs[t];
    }
    const int r_lane = wm * WTM + 4 * lhalf;   // first row of this lane inside the tile
    const int c_lane = wn * WTN + lcol;
    const bool full = (row0 + BM <= p.M) && (col0 + BN <= p.N);
    // what this lane's columns contribute to the requantization, fetched once ahead of the stores (columns past N
    // of the padded tile read the padded column sums and the first column's parameters; nothing of them is stored)
    RequantCol rqc[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        rqc[t].sub = 0;
        rqc[t].mult = 0.0f;
        if (kWantQ) {
            const int col = col0 + c_lane + t * 32;
            rqc[t] = requant_col(p.colsum[col], col < p.N ? col : 0, p.rq);
        }
    }
    const int32_t rq_zC = kWantQ ? p.rq.zC : 0;
    int32_t* cptr = kWantC ? p.C + (int64_t)(row0 + r_lane) * p.ldc + col0 + c_lane : nullptr;
    uint8_t* qptr = kWantQ ? p.Cq + (int64_t)(row0 + r_lane) * p.ldcq + col0 + c_lane : nullptr;
    const int rows_left = p.M - row0 - r_lane;  // rows of this lane's column that exist
    auto store_blocks = [&](auto full_c, auto mod_c, auto scatter_c) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_c)::value;  // no bounds to test inside a whole tile
        constexpr bool MOD = decltype(mod_c)::value;    // row sums as residues modulo 127 (Algorithm 1 as printed)
        // Cross-lane part of the row sums: the sixteen rows of a block together (sum32_of16), or one
        // reduction per row between the stores (see where the choice is made).
        constexpr bool kScatterSum = decltype(scatter_c)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            uint32_t rsv[16];  // this lane's part of the sixteen row sums of the block
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int ee = 0; ee < 4; ++ee) {
                    const int e = g * 4 + ee;
                    const int roff = i * 32 + 8 * g + ee;
                    uint32_t rs = (uint32_t)cs_lane;
                    long long rs64 = cs_lane64;  // exact sum for the residue (a wrapped sum would break it)
#pragma unroll
                    for (int t = 0; t < TN; ++t) {
                        const int32_t raw = acc[i][t][e];
                        if (kCheck && !MOD) rs += (uint32_t)raw;  // columns past N hold zeros
                        if (kCheck && MOD) rs64 += raw;
                        const int32_t val = raw + cs[t];
                        if (FULL || (roff < rows_left && col0 + c_lane + t * 32 < p.N)) {
                            if (kWantC) {
                                if (kAhead2) cptr[t * 32] = val;
                                else __builtin_nontemporal_store(val, &cptr[t * 32]);
                            }
                            if (kWantQ) qptr[t * 32] = requant_with(val, rqc[t], rq_zC);
                        }
                    }
                    if (kCheck) {
                        if (MOD) rs = (uint32_t)floor_mod127(rs64);
                        if (kScatterSum) {
                            rsv[e] = rs;
                        } else {
                            rs = sum32(rs);
                            if (lcol == 0) s_rs[wn * BM + wm * WTM + roff + 4 * lhalf] = (int32_t)rs;
                        }
                    }
                    if (kWantC) cptr += p.ldc;
                    if (kWantQ) qptr += p.ldcq;
                    asm volatile("" : "+v"(cptr), "+v"(qptr));
                }
                // rows 8g+4 .. 8g+7 belong to the other half-wave
                if (kWantC) cptr += 4 * p.ldc;
                if (kWantQ) qptr += 4 * p.ldcq;
            }
            if (kCheck && kScatterSum) {
                // lane lcol of each half-wave holds the sum of row e = bit-reversed low four bits of lcol
                const uint32_t tot = sum32_of16(rsv, lcol);
                const int e = ((lcol & 1) << 3) | ((lcol & 2) << 1) | ((lcol & 4) >> 1) | ((lcol & 8) >> 3);
                if (lcol < 16) s_rs[wn * BM + wm * WTM + i * 32 + 8 * (e >> 2) + (e & 3) + 4 * lhalf] = (int32_t)tot;
            }
        }
    };

    auto store_form = [&](auto full_c, auto mod_c) __attribute__((always_inline)) {
        store_blocks(full_c, mod_c, std::integral_constant<bool, kBlockSums>{});
    };
    if (mod127) {
        if (full) store_form(std::true_type{}, std::true_type{});
        else store_form(std::false_type{}, std::true_type{});
    } else {
        if (full) store_form(std::true_type{}, std::false_type{});
        else store_form(std::false_type{}, std::false_type{});
    }

    if (p.n_inj > 0) {
        // Simulated faults in the 32-bit intermediate (test hook): the element is flipped where it
        // now lies - in C, in Cq and in its row sum - by the lane that owns it, after that lane's
        // own store of the clean value (same lane, same address: program order holds).  The
        // accumulators are only read.  Entries that name the same element act as one entry
        // with the XOR of their masks.
        const abft_inject_t* inj = reinterpret_cast<const abft_inject_t*>(p.inj);
        for (int n = 0; n < p.n_inj; ++n) {
            const int row = inj[n].row, col = inj[n].col;
            const int r = row - (row0 + wm * WTM), c = col - (col0 + wn * WTN);
            if (r < 0 || r >= WTM || c < 0 || c >= WTN || row >= p.M || col >= p.N) continue;
            bool seen = false;
            for (int m = 0; m < n; ++m) seen |= (inj[m].row == row && inj[m].col == col);
            if (seen) continue;
            uint32_t mask = inj[n].xor_mask;
            for (int m = n + 1; m < p.n_inj; ++m)
                if (inj[m].row == row && inj[m].col == col) mask ^= inj[m].xor_mask;
            const int bi = r >> 5, rr = r & 31, bj = c >> 5;
            const int e_hit = (rr >> 3) * 4 + (rr & 3), half_hit = (rr >> 2) & 1;
            int32_t raw = 0, cs_hit = 0;
            RequantCol rqc_hit = rqc[0];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (i == bi && t == bj && e == e_hit) raw = acc[i][t][e];
#pragma unroll
            for (int t = 0; t < TN; ++t)
                if (t == bj) { cs_hit = cs[t]; rqc_hit = rqc[t]; }
            if (lcol == (c & 31) && lhalf == half_hit) {
                const int32_t val = raw + cs_hit, bad = (int32_t)((uint32_t)val ^ mask);
                if (kWantC) p.C[(int64_t)row * p.ldc + col] = bad;
                if (kWantQ) p.Cq[(int64_t)row * p.ldcq + col] = requant_with(bad, rqc_hit, rq_zC);
                // (the row sum was formed from the clean value; it is moved by the difference, taken in
                // wrap-around arithmetic: a flip of bit 31 changes the value by 2^31)
                if (kCheck)
                    atomicAdd(&s_rs[wn * BM + wm * WTM + r],
                              mod127 ? floor_mod127((long long)bad - val) : (int32_t)((uint32_t)bad - (uint32_t)val));
            }
        }
    }

    }  // if (last)

    if (kCheck) {
        // 16x16 accumulator: lane l, element e is row 4*(l/16) + e, column l%16; columns 0..3
        // hold the four digit products
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int d = lane & 15;
                uint32_t v = d < kLimbs ? ((uint32_t)cacc[c][e] << (8 * d)) : 0u;
                v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
                v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);
                if (d == 0) s_ck[wm * WTM + (wn * CB + c) * 16 + 4 * (lane >> 4) + e] = (int32_t)v;
            }
        __syncthreads();
        // Row r of the product is spread over the tile columns; each of them adds its share of
        // (row sum - checksum) to the row's 64-bit workspace word with ONE returned atomic:
        // the difference goes to the high half (it wraps there as int32 arithmetic does), an
        // arrival count to the low half.  The tile column that finds tiles_n - 1 arrivals before
        // it has the complete difference in hand: it writes the row's flag and clears the word.
        // No cache maintenance is involved: all data that crosses workgroups moves through
        // device-scope atomics.
        unsigned long long* const ws_rows = reinterpret_cast<unsigned long long*>(p.ws + kWsHeaderInts);
        static_assert(BM <= NT, "one row per thread at most");
        bool fin = false, bad = false;  // this thread completed its row / found it corrupted
        const int r = tid;
        if (r < BM && row0 + r < p.M) {
            uint32_t d = 0;
            if (last) {
#pragma unroll
                for (int w = 0; w < WGN; ++w) d += (uint32_t)s_rs[w * BM + r];
            }
            const bool first = tile_n == 0 && z == 0;   // the workgroup that accounts for the u8 -> s8 shift of the checksum product
            const int arrivals = tiles_n * Z;           // contributions a row's word receives
            if (mod127) {
                // residues: sums of at most 32 lanes x WGN waves of values below 127, minus the exact
                // checksum share, as a residue again so that the workspace word cannot wrap
                long long dd = (long long)d - (long long)s_ck[r];
                if (first) dd -= 128ll * (long long)total_sb;
                d = (uint32_t)floor_mod127(dd);
            } else {
                d -= (uint32_t)s_ck[r];
                if (first) d -= 128u * (uint32_t)total_sb;  // sum_k 128*S_B[k], once per row
            }
            if (arrivals == 1) {
                // one tile column holds the whole row: the comparison ends here, nothing crosses workgroups
                bad = mod127 ? (d % 127u != 0) : (d != 0);
                p.row_flags[row0 + r] = bad ? 1 : 0;
                fin = true;
            } else {
                const unsigned long long old = __hip_atomic_fetch_add(ws_rows + row0 + r, ((unsigned long long)d << 32) | 1ull,
                                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((uint32_t)old == (uint32_t)arrivals - 1u) {
                    const uint32_t diff = (uint32_t)(old >> 32) + d;
                    bad = mod127 ? (diff % 127u != 0) : (diff != 0);
                    __hip_atomic_store(ws_rows + row0 + r, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    p.row_flags[row0 + r] = bad ? 1 : 0;
                    fin = true;
                }
            }
        }
        // errCount: every row is completed by exactly one thread of the grid.  A wavefront that completed
        // rows reports them with one more returned atomic on the word of finished rows (count in the low
        // half, corrupted ones in the high half); the report that brings the count to M has the total,
        // writes errCount and clears the word.  Workgroups that completed nothing are done here, and no
        // barrier stands between the two atomics.
        // With p.err_accumulate the count is a counter that is added to: only wavefronts that found corrupted
        // rows touch it (one atomic without a return value), and nobody waits for anything.
        const unsigned long long fin_mask = __ballot(fin), bad_mask = __ballot(fin && bad);
        if (p.err_count == nullptr) {
            // no count was asked for
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
    // direct-to-LDS loads that are still in flight must not outlive the workgroup's LDS
    wait_vmem();
#ifdef ABFT_CLOCK_TRACE
    if (p.clock_trace && threadIdx.x == 0) {
        unsigned long long* const o = p.clock_trace + (size_t)blockIdx.x * 6;
        o[4] = clock64();
        o[5] = wall_clock64();
    }
#endif
}

template <int BM, int BN, int WGM, int WGN, int kStages, int WGK = 1, bool kSplitK = false>
hipError_t launch_cfg(bool check, bool want_c, bool want_q, const GemmParams& p_in, hipStream_t s) {
    GemmParams p = p_in;
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    int Z = 1;
    if (kSplitK) {
        // slices, tickets and partial tiles as splitk_plan lays them out; refused when the workspace does not hold them
        const SplitKPlan pl = splitk_plan(p.M, p.N, p.KB2);
        if (pl.z < 2 || p.ws == nullptr || p.ws_ints < pl.total_ints) return hipErrorNotSupported;
        Z = pl.z;
        p.ksplit = Z;
        p.ws_tickets = p.ws + pl.tickets_off;
        p.ws_part = p.ws + pl.part_off;
    }
    p.share_q = (p.KB2 / (WGK * Z)) / tiles_n;   // stages of the checksum product per tile column (and K group / slice)
    p.share_r = (p.KB2 / (WGK * Z)) % tiles_n;
    const dim3 grid((unsigned)(tiles_m * tiles_n * Z)), block(WGM * WGN * WGK * 64);
    const size_t lds = WGK * ((group_lds_bytes<BM, BN, WGN, kStages, WGK>() + 1023) / 1024 * 1024);
    if (WGK > 1) {
        // every group must pass the same barriers: equal runs of stages, and a share of the checksum
        // product that its staged digits hold without a refill (32 / WGK stages)
        const int ns = p.KB2;
        if (ns % WGK != 0 || ns / WGK < 2 || (ns / WGK + tiles_n - 1) / tiles_n > 32 / WGK) return hipErrorNotSupported;
    }
    // Row sums in block form or per row.  Small wave tiles: always the block form, which halves the
    // vector work of an epilogue that is short anyway.  The 128x128 wave tile: per row when the grid
    // fills the chip - the stores then take the time memory needs and the arithmetic between them is
    // hidden, while the sixteen extra live values of the block form cost registers the kernel does not
    // have (0.3 us slower at 4096^3) - and the block form when it does not: with fewer workgroups than
    // compute units the stores are not limited by memory and the arithmetic shows (3072^3: 45.0 us
    // per row, 42.4 us in block form).  Two kernels rather than a branch in one: with both forms in
    // one kernel the per-row form lost 1.7 us at 4096^3.
    constexpr bool kSmallWaveTile = (BM / WGM / 32) * (BN / WGN / 32) <= 4;
    const bool block_sums = kSmallWaveTile || grid.x < 256;
#define ABFT_LAUNCH(CK, OUT)                                                                              \
    do {                                                                                                  \
        if (block_sums) ABFT_LAUNCH_FORM(CK, OUT, true);                                                  \
        ABFT_LAUNCH_FORM(CK, OUT, (kSmallWaveTile || !(CK)));                                             \
    } while (0)
#define ABFT_LAUNCH_FORM(CK, OUT, BS)                                                                     \
    do {                                                                                                  \
        auto kern = gemm_tile_async_kernel<BM, BN, WGM, WGN, kStages, CK, OUT, ((BS) || !(CK)), WGK, kSplitK>; \
        static std::atomic<uint64_t> lds_allowed{0};                                                      \
        const hipError_t e_attr = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds, lds_allowed);\
        if (e_attr != hipSuccess) return e_attr;                                                          \
        kern<<<grid, block, lds, s>>>(p, tiles_m, tiles_n);                                               \
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
#undef ABFT_LAUNCH_FORM
}

}  // namespace atile
}  // namespace abft
