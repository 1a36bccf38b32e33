// Persistent grouped bf16 GEMM in which the two waves of every SIMD take turns at the matrix pipe
// (sbp_matmul, paper Sec. 3.1, Table 1: device g computes C_g = A_g B_g).
//
// 256 x 256 output tile per workgroup, 8 waves of 128 x 64, v_mfma_f32_16x16x32_bf16, four 32-deep LDS
// stages filled by direct-to-LDS loads, one persistent workgroup per compute unit that walks many
// tiles: as in gemm_mfma_persist16_kernel.  What differs:
//
// (1) Ping-pong.  A wave that reads its operand fragments from LDS between its matrix instructions
//     issues those at well below the pipe's rate (measured on gfx950: 64 instructions of two waves
//     take 1270-1720 cycles with 8-16 fragment reads among each wave's 32, 1056 with none), and when
//     both waves of a SIMD do the same thing at the same time nobody fills the gaps.  Here the waves
//     0-3 (one per SIMD, upper 128 rows of the tile) and 4-7 (lower 128 rows) run ONE PHASE APART:
//         waves 0-3:  load(s)   | compute(s) | load(s+1)  | compute(s+1) | ...
//         waves 4-7:  compute(s-1) | load(s) | compute(s) | load(s+1)    | ...
//     with a workgroup barrier between phases.  load(s): all fragments of reduction step s, LDS ->
//     registers (48 registers; they need no second set, the wave does not compute meanwhile), then the
//     direct-to-LDS loads of stage s + 3: waves 0-3 bring the X tile, waves 4-7 the W tile.
//     compute(s): 32 matrix instructions back to back.  The pipe always has exactly one wave feeding it.
//     A stage is read during two consecutive phases only, so four stages keep the loads three steps ahead.
//
// (2) The matrix instruction is fed (W fragment, X fragment), so that a lane's four accumulator
//     registers of a 16 x 16 block hold four consecutive COLUMNS of one output row (row = lane % 16,
//     columns 4 (lane / 16) + 0..3) and enter the epilogue's LDS window as one 16-byte (bf16: 8-byte)
//     write per block instead of four 4-byte ones.  The window (4 KB per wave, private, no workgroup
//     barrier) turns the results so that eight CONSECUTIVE lanes own the eight 16-byte chunks of one
//     128-byte line: the store path merges only neighbouring lanes (measured: 16-byte pieces of a line
//     held by lanes 16 apart store at half the rate of the same bytes held by neighbours, however the
//     pieces are arranged in memory).
//     A group stores its half of a finished tile at the start of its next load phase, i.e. while the
//     other group still computes; the two epilogues of a tile do not coincide.
//
// (3) The fused row maximum (sbp_matmul_rowmax, Sec. 6.3.1) is carried in registers from tile to tile while the
//     tile walk stays in the same rows and reaches the P(max) vector only when the rows change (see runpk).
//
// Registers: 128 accumulators + 48 fragment registers of 256, and the unrolled four-stage loop needs most of the
// rest for LDS addresses; whatever is only needed at a tile change (lane id and everything derived from it) is
// recomputed there.  A spill would be more than a slow access: its reload waits for the whole memory counter.
//
// Loads and stores are inline assembly outside the compiler's bookkeeping (see gemm_device.h) and every
// wait on the memory counter is explicit.  The counter retires in issue order.  Before the barrier that
// opens load(s + 1) of waves 0-3 (the first reader of stage s + 1) every wave waits for its part of that
// stage: waves 0-3 at the end of compute(s), waves 4-7 at the end of their load(s); "all but the two
// youngest stages", plus the stores of a tile's epilogue while those are younger than the stage (the
// first two steps of the next tile).
#include "gemm_device.h"

namespace sbp {
namespace {

template <int V> using ic = std::integral_constant<int, V>;
constexpr int vm_lgkm0(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070; }   // s_waitcnt vmcnt(n) lgkmcnt(0)
constexpr int LGKM0 = 0xC07F;                                                     // s_waitcnt lgkmcnt(0), vmcnt untouched

// 16-byte store at (uniform base) + (per-lane 32-bit byte offset) + IMM, untracked.  The idle cycles cover the
// rule that the data registers of a wide store must not be rewritten right behind it.
template <int IMM, typename V>
__device__ inline void store16_sbase(const char* base, uint32_t voff, const V v, bool stream) {
    if (stream) asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3 nt\n\ts_nop 1" : : "v"(voff), "v"(v), "s"(base), "n"(IMM) : "memory");
    else asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3\n\ts_nop 1" : : "v"(voff), "v"(v), "s"(base), "n"(IMM) : "memory");
}

// global -> LDS without passing through registers, untracked: lane i's 16 bytes land at (base + IMM) + 16 i.  M0
// carries that LDS address; one idle cycle separates its write from the load that reads it.
template <int IMM>
__device__ inline void load16_lds(uint32_t lds_base, gbl_char* src, uint32_t voff) {
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(src), "s"(lds_base), "n"(IMM) : "memory", "m0", "scc");
}
// The same load marked non-temporal: for an operand whose tiles are read at one time only (the caches need not keep them).
template <int IMM>
__device__ inline void load16_lds_stream(uint32_t lds_base, gbl_char* src, uint32_t voff) {
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" : : "v"(voff), "s"(src), "s"(lds_base), "n"(IMM) : "memory", "m0", "scc");
}

// the part of an output tile that one wave writes (all uniform)
struct OutTile {
    char* base;        // element (m0 + wm * 128, n0 + wn * 64)
    uint32_t rowblk;   // bytes between row blocks (16 rows)
    int32_t ldc;
    bool stream;       // row pitch a multiple of 128 bytes: whole lines, stored past the cache
    bool whole;        // not cut by the matrix edge, rows 16-byte aligned
    int32_t rows_left, cols_left;   // of the matrix, from the wave tile's first row / column on
    int32_t rows_key;               // (shard << 16 | tile row) + 1: names the rows this wave writes
};

template <bool A_KC, bool B_KC, int EPI, typename OutT>
__global__ __launch_bounds__(512) void gemm_pingpong_kernel(GemmPlan p, int tm, int tn, int order, int nblk) {
    constexpr int BM = 256, BN = 256, NTL = 256, BKT = 32, TM = 128, TN = 64;
    constexpr bool F32OUT = sizeof(OutT) == 4;
    using TA = Tile<BM, A_KC, NTL, BKT, true>;      // loaded by the 256 threads of waves 0-3
    using TB = Tile<BN, B_KC, NTL, BKT, true>;
    static_assert(TA::PER_THREAD == TB::PER_THREAD, "both groups issue the same number of loads");
    constexpr int NL = TA::PER_THREAD;                                           // loads per stage and wave (4)
    constexpr int NSW = F32OUT ? 32 : 16;                                        // stores per tile and wave
    static_assert(2 * NL + NSW < 64, "vmcnt field");
    // four stages in one array (stage b: X tile at b * STAGE, W tile behind it), so that every LDS address a
    // load needs is one scalar base plus an immediate
    constexpr int STAGE = TA::BYTES + TB::BYTES;
    __shared__ __attribute__((aligned(1024))) char smem[4 * STAGE];
    __shared__ __attribute__((aligned(1024))) char swin[8 * 4096];   // epilogue windows, one per wave
    auto stA = [&](auto i) -> char* { return smem + decltype(i)::value * STAGE; };
    auto stB = [&](auto i) -> char* { return smem + decltype(i)::value * STAGE + TA::BYTES; };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the lane id again, from the hardware and opaque to the compiler: what the epilogue and the tile changes derive
    // from it is recomputed there instead of occupying a register all through the reduction loop, which has none to spare
    auto lane_again = []() {
        int l;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
        return l;
    };
    // Bit 16 of `order`: every tile row of a shard lies in one band of the walk, so a W tile is wanted by the workgroups
    // of that band at one time and never again: its loads are marked non-temporal (measured on the classifier logits,
    // 4 tile rows x 489 tile columns per shard: 3-4 % faster; with W tiles that later bands read again, 33 % slower).
    const bool w_stream = (order >> 16) & 1;
    order &= 0xFFFF;
    const int grp = wave >> 2;            // 0: loads operands and runs one phase ahead; 1: one phase behind
    const int wm = grp, wn = wave & 3;
    const int G = gridDim.x;

    // first valid tile at or after virtual block v (uneven shards have fewer tiles than tm x tn)
    auto next_valid = [&](int v) {
        for (; v < nblk; v += G) {
            const TileCoord tc = map_tile(v, nblk, tm, tn, p.groups, order);
            if (tc.valid && tc.tile_m * BM < p.s[tc.g].m && tc.tile_n * BN < p.s[tc.g].n) break;
        }
        return v;
    };
    const int first = next_valid(blockIdx.x);
    if (first >= nblk) return;

    // ---- load cursor (waves 0-3): stage after stage, tile after tile, three steps ahead of compute ----
    gbl_char* A = nullptr;
    gbl_char* B = nullptr;
    uint32_t off[NL];          // per-lane source offsets of this wave's loads: of the X tile in waves 0-3, of the W tile in waves 4-7
    uint32_t stepa = 0, stepb = 0;
    auto open_tile = [&](int v) {
        const TileCoord tc = map_tile(v, nblk, tm, tn, p.groups, order);
        const GemmShard& s = p.s[tc.g];
        A = (gbl_char*)s.a;
        B = (gbl_char*)s.b;
        const int t = (wave & 3) * 64 + lane_again();   // thread index within the four waves that load this operand
        if (grp == 0) {
#pragma unroll
            for (int it = 0; it < NL; ++it) off[it] = TA::src_offset(s.lda, tc.tile_m * BM, s.m, it * NTL + t);
        } else {
#pragma unroll
            for (int it = 0; it < NL; ++it) off[it] = TB::src_offset(s.ldb, tc.tile_n * BN, s.n, it * NTL + t);
        }
        stepa = TA::step_bytes(s.lda);
        stepb = TB::step_bytes(s.ldb);
    };
    // always NL loads (the wait counts rely on it), then one stage forward.  Every wave keeps the whole cursor
    // (it is uniform scalar state); waves 0-3 load the X tile of a stage, waves 4-7 its W tile.
    const uint32_t lds_wave = (uint32_t)(uintptr_t)(lds_void*)smem + (uint32_t)wn * 1024u;   // this wave's 64 chunks of a 256-chunk row of loads
    auto issue = [&](auto dst) {
        constexpr int D = decltype(dst)::value;
        if (grp == 0) static_for<NL>([&](auto it) { load16_lds<D * STAGE + decltype(it)::value * NTL * 16>(lds_wave, A, off[decltype(it)::value]); });
        else if (w_stream) static_for<NL>([&](auto it) { load16_lds_stream<D * STAGE + TA::BYTES + decltype(it)::value * NTL * 16>(lds_wave, B, off[decltype(it)::value]); });
        else static_for<NL>([&](auto it) { load16_lds<D * STAGE + TA::BYTES + decltype(it)::value * NTL * 16>(lds_wave, B, off[decltype(it)::value]); });
        A += stepa;
        B += stepb;
    };

    // ---- registers -------------------------------------------------------------------------------
    // acc[i][j]: lane l holds C[16 i + l % 16][16 j + 4 (l / 16) + 0..3] of the wave tile
    f32x4 acc[8][4];
    bf16x8 fa[8], fb[4];
    const int loa = TA::lane_offset16(wm * TM, lane), lob = TB::lane_offset16(wn * TN, lane);
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};

    // ---- epilogue --------------------------------------------------------------------------------
    // Window of a wave: fp32 one row block (16 rows x 256 B), bf16 two (16 rows x 128 B each).  Lane (g, c) =
    // (lane / 16, lane % 16) writes its row c; lane l reads row l / 8 (+ 8), 16-byte chunk l % 8 (+ 8).  The chunks of
    // a row are permuted so that neither side has a bank conflict:
    //   fp32 (16 chunks per row, a row spans all banks): chunk ^ (8 (row & 1) | (row >> 1) & 7).  The 16 lanes of a
    //        write pass hold 16 rows: 16 different chunks; the 16 lanes of a read pass hold two neighbouring rows, 8
    //        chunks each: the rows differ in bit 3 of the permutation, so again 16 different chunks.
    //   bf16 (8 chunks per row, two rows span the banks): chunk ^ ((row >> 1) & 7).  A write pass (8 bytes per lane):
    //        the eight even rows take eight different chunks in one half of the banks, the odd rows in the other;
    //        a read pass: two neighbouring rows, same permutation, different halves.
    // EPI_ROWMAX (Sec. 6.3.1, local row maximum): lane (g, c) keeps, for each of its 8 row blocks i, the maximum of the
    // values it has stored of row 16 i + c (its columns 16 j + 4 g + 0..3 of every tile), carried from tile to tile while
    // the tile walk stays in the same rows: one max3 per two values per tile, plus unpacking and repacking the eight
    // running values, which are kept as bf16 pairs in four registers (eight would not stay in registers across the
    // reduction loop, and a spill brings the compiler's own full wait on the memory counter into every tile).  Only when the rows change
    // or the kernel ends do the four lanes of a row combine (two lane swaps) and one pair of atomics per 64 rows fold
    // the result into the P(max) vector: a shard's column tiles would otherwise all send atomics to the same few cache
    // lines.  The maximum is taken over the fp32 results and rounded once: rounding to nearest even is monotonic, so
    // that is the maximum of the stored bf16 values.  The extra memory operations of a flush only make the counted
    // waits behind it stricter.
    [[maybe_unused]] uint32_t runpk[4];      // row blocks 2 q (low half) and 2 q + 1 (high half), bf16
    [[maybe_unused]] int run_key = 0;        // OutTile::rows_key of the rows the running maxima belong to, 0 = none yet (uniform)
    if constexpr (EPI == EPI_ROWMAX) {
#pragma unroll
        for (int q = 0; q < 4; ++q) runpk[q] = 0xFF80FF80u;   // -inf, -inf
    }
    [[maybe_unused]] auto flush_rowmax = [&]() {
        const int ln = lane_again();
        const int g = ln >> 4;
        const GemmShard& rs = p.s[(run_key - 1) >> 16];
        const int first_row = ((run_key - 1) & 0xFFFF) * BM + wm * TM;
        float* run_ptr = rs.rowmax + first_row;
        const int run_rows = rs.m - first_row;      // 128 or more: all of the wave's rows exist
        float r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t x = (i & 1) ? (runpk[i >> 1] & 0xFFFF0000u) : (runpk[i >> 1] << 16);
            const auto a = __builtin_amdgcn_permlane32_swap(x, x, false, false);
            const uint32_t m = __float_as_uint(max3f(__uint_as_float(a[0]), __uint_as_float(a[1]), __uint_as_float(a[1])));
            const auto b = __builtin_amdgcn_permlane16_swap(m, m, false, false);
            r[i] = max3f(__uint_as_float(b[0]), __uint_as_float(b[1]), __uint_as_float(b[1]));
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) runpk[q] = 0xFF80FF80u;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // lane 16 g + c carries row 64 h + 16 g + c, i.e. row c of row block 4 h + g
            float vmax = g == 0 ? r[4 * h] : g == 1 ? r[4 * h + 1] : g == 2 ? r[4 * h + 2] : r[4 * h + 3];
            vmax = bf16_to_f32(f32_to_bf16(vmax)) + 0.0f;
            float* dst = run_ptr + h * 64 + ln;
            const bool row_ok = h * 64 + ln < run_rows;
            // signed max for non-negative values, unsigned min for negative ones (see atomic_max_f32_untracked), each
            // under its own lanes; a NaN never entered the running maximum
            const uint64_t mp = __builtin_amdgcn_ballot_w64(row_ok && vmax >= 0.0f), mn = __builtin_amdgcn_ballot_w64(row_ok && vmax < 0.0f);
            asm volatile("s_mov_b64 exec, %2\n\tglobal_atomic_smax %0, %1, off\n\ts_mov_b64 exec, %3\n\tglobal_atomic_umin %0, %1, off\n\ts_mov_b64 exec, -1"
                         : : "v"(dst), "v"(vmax), "s"(mp), "s"(mn) : "memory");
        }
    };

    auto store_tile = [&](const OutTile& ot) {
        const int ln = lane_again();
        const int g = ln >> 4, c = ln & 15;
        if constexpr (EPI == EPI_ROWMAX) {
            if (run_key != ot.rows_key) {            // uniform: other rows than the running maxima belong to
                if (run_key) flush_rowmax();
                run_key = ot.rows_key;
            }
        }
        if (ot.whole) {
            char* win = swin + wave * 4096;
            const int rr = ln >> 3, rk = ln & 7;           // read side: row (of 8), chunk (of 8)
            if constexpr (F32OUT) {
                const int wbase = c * 256 + ((g ^ (8 * (c & 1)) ^ ((c >> 1) & 7)) << 4);      // block j adds (4 j) to the chunk: an XOR of bits 2, 3
                int rd[2][2];   // [row half t][line half h]
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int row = 8 * tt + rr;
                        rd[tt][h] = row * 256 + (((8 * h + rk) ^ (8 * (row & 1)) ^ ((row >> 1) & 7)) << 4);
                    }
                const uint32_t vofs = (uint32_t)(rr * ot.ldc) * 4u + (uint32_t)rk * 16u;
                static_for<8>([&](auto idx) {
                    constexpr int IA = decltype(idx)::value;
#pragma unroll
                    for (int j = 0; j < 4; ++j) *reinterpret_cast<f32x4*>(win + (wbase ^ (j << 6))) = acc[IA][j];
                    __builtin_amdgcn_wave_barrier();
                    const char* rb = ot.base + (size_t)IA * ot.rowblk;
                    static_for<4>([&](auto q) {
                        constexpr int T = decltype(q)::value / 2, H = decltype(q)::value % 2;
                        const u32x4 v = *reinterpret_cast<const u32x4*>(win + rd[T][H]);
                        store16_sbase<H * 128>(rb + (T ? (ot.rowblk >> 1) : 0), vofs, v, ot.stream);
                    });
                    __builtin_amdgcn_wave_barrier();
                });
            } else {
                // rounded to bf16, lane (g, c) holds columns 4 g + 0..3 of block j as two dwords: bytes 32 j + 8 g of its row
                const int wbase = c * 128 + ((((g >> 1)) ^ ((c >> 1) & 7)) << 4) + (g & 1) * 8;   // block j adds (2 j) to the chunk: an XOR of bits 1, 2
                int rd[2];
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    const int row = 8 * tt + rr;
                    rd[tt] = row * 128 + ((rk ^ ((row >> 1) & 7)) << 4);
                }
                const uint32_t vofs = (uint32_t)(rr * ot.ldc) * 2u + (uint32_t)rk * 16u;
                static_for<4>([&](auto idx) {
                    constexpr int IP = decltype(idx)::value;      // row blocks 2 IP, 2 IP + 1 share the window
                    [[maybe_unused]] float pairmx[2];
                    static_for<2>([&](auto sub) {
                        constexpr int IA = 2 * IP + decltype(sub)::value;
                        [[maybe_unused]] float mx = 0.0f;
                        if constexpr (EPI == EPI_ROWMAX) mx = __uint_as_float((IA & 1) ? (runpk[IP] & 0xFFFF0000u) : (runpk[IP] << 16));
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float v0 = mfma_epilogue<EPI>(acc[IA][j][0]), v1 = mfma_epilogue<EPI>(acc[IA][j][1]);
                            const float v2 = mfma_epilogue<EPI>(acc[IA][j][2]), v3 = mfma_epilogue<EPI>(acc[IA][j][3]);
                            if constexpr (EPI == EPI_ROWMAX) mx = max3f(max3f(mx, v0, v1), v2, v3);
                            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                            const u32x2 w = {f32_to_bf16x2(v0, v1), f32_to_bf16x2(v2, v3)};
                            *reinterpret_cast<u32x2*>(win + (decltype(sub)::value * 2048 + (wbase ^ (j << 5)))) = w;
                        }
                        if constexpr (EPI == EPI_ROWMAX) pairmx[IA & 1] = mx;
                    });
                    if constexpr (EPI == EPI_ROWMAX) runpk[IP] = f32_to_bf16x2(pairmx[0], pairmx[1]);
                    __builtin_amdgcn_wave_barrier();
                    static_for<4>([&](auto q) {
                        constexpr int SUB = decltype(q)::value / 2, T = decltype(q)::value % 2, IA = 2 * IP + SUB;
                        const u32x4 v = *reinterpret_cast<const u32x4*>(win + (SUB * 2048 + rd[T]));
                        store16_sbase<0>(ot.base + (size_t)IA * ot.rowblk + (T ? (ot.rowblk >> 1) : 0), vofs, v, ot.stream);
                    });
                    __builtin_amdgcn_wave_barrier();
                });
            }
            return;
        }
        // tiles cut by the matrix edge or with unaligned rows: element by element, guarded, then a full drain
        OutT* C = reinterpret_cast<OutT*>(ot.base);
        [[maybe_unused]] float runmax[8];
        if constexpr (EPI == EPI_ROWMAX) {
#pragma unroll
            for (int q = 0; q < 8; ++q) runmax[q] = __uint_as_float((q & 1) ? (runpk[q >> 1] & 0xFFFF0000u) : (runpk[q >> 1] << 16));
        }
        static_for<32>([&](auto idx) {
            constexpr int i = decltype(idx)::value / 4, j = decltype(idx)::value % 4;
            const int m = 16 * i + c;
            const int nb = 16 * j + 4 * g;
            OutT* cp = C + (int64_t)m * ot.ldc + nb;
            static_for<4>([&](auto ridx) {
                constexpr int r = decltype(ridx)::value;
                const float v = mfma_epilogue<EPI>(acc[i][j][r]);
                if (m < ot.rows_left && nb + r < ot.cols_left) store_out_untracked(cp, (int64_t)r, v);
                // columns past the matrix edge stay out of the row maximum; rows past it are masked when it is flushed
                if constexpr (EPI == EPI_ROWMAX) runmax[i] = max3f(runmax[i], nb + r < ot.cols_left ? v : -__builtin_inff(), -__builtin_inff());
            });
        });
        if constexpr (EPI == EPI_ROWMAX) {
#pragma unroll
            for (int q = 0; q < 4; ++q) runpk[q] = f32_to_bf16x2(runmax[2 * q], runmax[2 * q + 1]);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    };

    // ---- one reduction step: load phase, barrier, compute phase, barrier -------------------------
    // BUF: LDS stage of this step.  ZERO: first step of a tile (the accumulators start from zero).
    // stores_young (uniform, waves 0-3): the stores of the previous tile's epilogue were issued after the stage
    // that this step's final wait is about.
    auto step = [&](auto buf, auto zero, bool stores_young) {
        constexpr int BUF = decltype(buf)::value;
        constexpr bool ZERO = decltype(zero)::value;
        using DST = ic<(BUF + 3) % 4>;
#pragma unroll
        for (int j = 0; j < 4; ++j) fb[j] = TB::frag16(stB(buf), lob, j);
#pragma unroll
        for (int i = 0; i < 8; ++i) fa[i] = TA::frag16(stA(buf), loa, i);
        __builtin_amdgcn_sched_barrier(0);
        issue(DST{});                                     // this group's tile of stage s + 3, underneath the LDS latency
        if (grp == 1) {
            // waves 4-7: their part of stage s + 1 has landed (all but the two youngest stages)
            if (stores_young) __builtin_amdgcn_s_waitcnt(vm_lgkm0(2 * NL + NSW));
            else __builtin_amdgcn_s_waitcnt(vm_lgkm0(2 * NL));
        } else {
            __builtin_amdgcn_s_waitcnt(LGKM0);
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (ZERO) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], zero4, 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
            }
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        if (grp == 0) {
            // waves 0-3: their part of stage s + 1 has landed
            if (stores_young) __builtin_amdgcn_s_waitcnt(vmcnt_only(2 * NL + NSW));
            else __builtin_amdgcn_s_waitcnt(vmcnt_only(2 * NL));
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };

    auto out_tile = [&](const TileCoord& tc) {
        const GemmShard& s = p.s[tc.g];
        const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
        constexpr int EPV = 16 / (int)sizeof(OutT);
        OutTile ot;
        ot.base = static_cast<char*>(s.c) + ((int64_t)(m0 + wm * TM) * s.ldc + (n0 + wn * TN)) * (int64_t)sizeof(OutT);
        ot.rowblk = (uint32_t)s.ldc * (16u * (uint32_t)sizeof(OutT));
        ot.ldc = s.ldc;
        ot.stream = ((int64_t)s.ldc * (int64_t)sizeof(OutT)) % 128 == 0;
        ot.whole = m0 + BM <= s.m && n0 + BN <= s.n && s.ldc % EPV == 0;
        ot.rows_left = s.m - (m0 + wm * TM);
        ot.cols_left = s.n - (n0 + wn * TN);
        ot.rows_key = __builtin_amdgcn_readfirstlane(((tc.g << 16) | tc.tile_m) + 1);
        return ot;
    };

    // stages 0, 1, 2 of the first tile; step 0 issues stage 3
    open_tile(first);
    static_for<3>([&](auto i) { issue(i); });
    __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (grp == 1) __builtin_amdgcn_s_barrier();   // waves 4-7 run one phase behind

    bool pend = false;     // the previous tile is still in the accumulators
    OutTile prev{};
    for (int cv = first; cv < nblk;) {
        const TileCoord tc = map_tile(cv, nblk, tm, tn, p.groups, order);
        const int rounds = p.s[tc.g].kk / (BKT * 4);
        const int nv = next_valid(cv + G);
        // the load cursor has issued this tile's last stage: move it to the next tile
        auto switch_tile = [&]() {
            if (nv < nblk) {
                open_tile(nv);
            } else {
                A -= stepa;     // no next tile: keep re-reading the last stage
                B -= stepb;
                stepa = 0;
                stepb = 0;
            }
        };
        // the finished tile leaves at the start of this group's load phase, while the other group computes
        bool young = false;
        if (pend) {
            store_tile(prev);
            young = prev.whole;
        }
        step(ic<0>{}, std::true_type{}, young);
        if (rounds == 1) switch_tile();
        step(ic<1>{}, std::false_type{}, young);
        step(ic<2>{}, std::false_type{}, false);
        step(ic<3>{}, std::false_type{}, false);
        for (int r = 1; r < rounds; ++r) {
            step(ic<0>{}, std::false_type{}, false);
            if (r == rounds - 1) switch_tile();
            step(ic<1>{}, std::false_type{}, false);
            step(ic<2>{}, std::false_type{}, false);
            step(ic<3>{}, std::false_type{}, false);
        }
        pend = true;
        prev = out_tile(tc);
        cv = nv;
    }
    if (pend) store_tile(prev);
    if constexpr (EPI == EPI_ROWMAX) {
        if (run_key) flush_rowmax();
    }
    if (grp == 0) __builtin_amdgcn_s_barrier();   // pairs with the last barrier of waves 4-7
    __builtin_amdgcn_s_waitcnt(0x0070);           // trailing loads must land before LDS is released; stores drain
}

template <bool A_KC, bool B_KC>
int32_t launch_pp_cfg(const GemmPlan& plan, int tm, int tn, int order, int nblk, int grid, hipStream_t st) {
    if (plan.out_dtype == SBP_F32)
        hipLaunchKernelGGL((gemm_pingpong_kernel<A_KC, B_KC, SBP_EPI_NONE, float>), dim3((uint32_t)grid), dim3(512), 0, st, plan, tm, tn, order, nblk);
    else if (plan.epilogue == SBP_EPI_GELU)
        hipLaunchKernelGGL((gemm_pingpong_kernel<A_KC, B_KC, SBP_EPI_GELU, uint16_t>), dim3((uint32_t)grid), dim3(512), 0, st, plan, tm, tn, order, nblk);
    else if (plan.epilogue == EPI_ROWMAX)
        hipLaunchKernelGGL((gemm_pingpong_kernel<A_KC, B_KC, EPI_ROWMAX, uint16_t>), dim3((uint32_t)grid), dim3(512), 0, st, plan, tm, tn, order, nblk);
    else
        hipLaunchKernelGGL((gemm_pingpong_kernel<A_KC, B_KC, SBP_EPI_NONE, uint16_t>), dim3((uint32_t)grid), dim3(512), 0, st, plan, tm, tn, order, nblk);
    return launch_status(__func__);
}

}  // namespace


// bf16 operands, every local reduction length a multiple of 128, row pitches of 16 bytes: checked by the caller
int32_t launch_gemm_pingpong(const GemmPlan& plan, int max_m, int max_n, int order, hipStream_t st) {
    const int tm = (max_m + 255) / 256, tn = (max_n + 255) / 256;
    const int64_t tiles = (int64_t)tm * tn * plan.groups;
    const int64_t nblk = (tiles + 7) / 8 * 8;
    if (nblk > 0x7FFFFFFF) return SBP_ERR_UNSUPPORTED;
    if (plan.out_dtype == SBP_F32 && plan.epilogue != SBP_EPI_NONE) return SBP_ERR_UNSUPPORTED;
    int grid = compute_units() / 8 * 8;
    if (grid > nblk) grid = (int)nblk;
    if (tm <= (order & 0xFF)) order |= 1 << 16;   // one band holds every tile row: W tiles are read at one time only
    if (plan.a_kc && plan.b_kc) return launch_pp_cfg<true, true>(plan, tm, tn, order, (int)nblk, grid, st);
    if (plan.a_kc) return launch_pp_cfg<true, false>(plan, tm, tn, order, (int)nblk, grid, st);
    if (plan.b_kc) return launch_pp_cfg<false, true>(plan, tm, tn, order, (int)nblk, grid, st);
    return launch_pp_cfg<false, false>(plan, tm, tn, order, (int)nblk, grid, st);
}

}  // namespace sbp
