// Grouped per-shard GEMM for sbp_matmul (paper Sec. 3.1, Table 1): device g computes
// C_g = A_g B_g from the local tensors it holds; all k devices run in ONE launch.
//
//   gemm_generic_kernel       any dtype / shape / pitch, one output element per lane, fp32 FMA chain.
//                             Used for fp32 operands and for shapes the MFMA kernels do not take.
//   gemm_mfma_kernel          bf16 x bf16 -> fp32 on the matrix cores (v_mfma_f32_32x32x16_bf16),
//                             BM x BN macro-tile per workgroup, global->LDS loads that bypass
//                             registers, two LDS stages of 64 reduction elements.
//   gemm_mfma_pipe_kernel     the same with 3-5 stages of 32 and partial waits on the load counter.
//   gemm_mfma_pipe16_kernel   four stages of 32 on v_mfma_f32_16x16x32_bf16: large shapes whose reduction
//                             length is a multiple of 64 but not of 128.
//   gemm_mfma_persist_kernel  four stages, one workgroup per compute unit walking many tiles, the next
//                             tile's loads in flight across the epilogue.
//   gemm_mfma_persist16_kernel  the same on v_mfma_f32_16x16x32_bf16 (store_tile16): the default for
//                             large shapes; under real operands the chip clocks this instruction higher.
//   gemm_split_kernel         one fp32 operand (a P(sum) partial) split exactly into three bf16 terms.
// All MFMA kernels share Tile (LDS images, swizzles, fragment reads) and store_tile (epilogue).
//
// Operand storage: "KC" = reduction index contiguous ([m][kk] for A, [n][kk] for B), otherwise the
// reduction index is the slow one ([kk][m], [kk][n]).  Row-major X and W give A KC and B not-KC.
#include <atomic>
#include <cstdlib>
#include <utility>

#include "sbp_internal.h"
#include "gemm_device.h"

namespace sbp {
namespace {

// 0.5 x (1 + erf(x / sqrt 2)) written with erfc so that the negative tail keeps its relative accuracy
__device__ inline float gelu_erf(float x) { return 0.5f * x * erfcf(x * -0.70710678118654752f); }

template <int EPI>
__device__ inline float epilogue(float v) {
    if constexpr (EPI == SBP_EPI_GELU) return gelu_erf(v);
    else return v;
}

// results are written once and not read again by this kernel: streaming (non-temporal) stores keep
// them from displacing operand tiles in L2
__device__ inline void store_out(float* c, int64_t pos, float v) {
    __builtin_nontemporal_store(v, c + pos);
}
__device__ inline void store_out(uint16_t* c, int64_t pos, float v) {
    __builtin_nontemporal_store(f32_to_bf16(v), c + pos);
}

// ------------------------------------------------------------------------------------------------
// generic kernel
// ------------------------------------------------------------------------------------------------
// A_BF16 / B_BF16: element type of each operand (a P(sum) operand is fp32 next to a bf16 one)
template <bool A_BF16, bool B_BF16, typename OutT, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmPlan p) {
    const GemmShard s = p.s[blockIdx.z];
    const int m = blockIdx.y * 16 + threadIdx.y;
    const int n = blockIdx.x * 16 + threadIdx.x;
    if (m >= s.m || n >= s.n) return;
    float acc = 0.0f;
    for (int kk = 0; kk < s.kk; ++kk) {
        const int64_t ia = p.a_kc ? (int64_t)m * s.lda + kk : (int64_t)kk * s.lda + m;
        const int64_t ib = p.b_kc ? (int64_t)n * s.ldb + kk : (int64_t)kk * s.ldb + n;
        float a, b;
        if constexpr (A_BF16) a = bf16_to_f32(static_cast<const uint16_t*>(s.a)[ia]);
        else a = static_cast<const float*>(s.a)[ia];
        if constexpr (B_BF16) b = bf16_to_f32(static_cast<const uint16_t*>(s.b)[ib]);
        else b = static_cast<const float*>(s.b)[ib];
        acc = fmaf(a, b, acc);
    }
    store_out(static_cast<OutT*>(s.c), (int64_t)m * s.ldc + n, epilogue<EPI>(acc));
}

// ------------------------------------------------------------------------------------------------
// MFMA kernel
// ------------------------------------------------------------------------------------------------


// tile walk: low byte = tile-rows per band (0 = chosen from the shape, see tile_order_for), bit 8 = skip
// the XCD re-linearisation
std::atomic<int> g_tile_order{0};

// Band height when the knob leaves it open.  Measured with the persistent kernels, ms at band
// 1 / 2 / 3 / 4 / 6 / 8 / 16: 32 x 8 tiles per shard (K = 4096) .815 / .809 / .805 / .812 / .828 / .844 / .932;
// 32 x 16 tiles (K = 2048 per shard) .947 / .945 / .906 / .905 / .897 / .900 / 1.18; 4 x 489 tiles: 3 or 4.
// So 2 for narrow shards, 6 for wide ones with enough tile-rows to fill whole bands, else 3; 4 for four tile-rows: a
// workgroup of the persistent walk then stays in the same rows from tile to tile (256 is a multiple of the band),
// which the fused row maximum uses.
inline int tile_order_for(int tm, int tn) {
    const int knob = g_tile_order.load(std::memory_order_relaxed);
    if (knob & 0xFF) return knob;
    return (knob & ~0xFF) | (tn <= 8 ? 2 : tm >= 12 ? 6 : tm == 4 ? 4 : 3);
}



// Epilogue of the MFMA kernels.  A wave's accumulators hold D[8 (r / 4) + 4 (lane / 32) + r % 4][lane % 32]
// = acc[r] for every 32 x 32 block: one column per lane.  Stored straight from there, a store
// instruction would write 4 bytes (fp32) or 2 bytes (bf16) per lane, two short row segments at a time;
// the memory pipeline takes 128 of those per wave and tile badly (with bf16 results and a short
// reduction the epilogue then costs more than the multiplication).  Instead every wave passes its
// results through a private 4 KB LDS window (STAGE_BYTES per wave, no workgroup barrier needed) that
// turns them by 90 degrees: each lane then owns 16 consecutive bytes of a row, and one store
// instruction writes eight complete 128-byte row segments.
//   fp32: one 32 x 32 block at a time, row pitch 128 B.  Row R is kept at R ^ ((R >> 2) & 1): the two
//         half-waves write rows R and R + 4 in one instruction and so land in different bank halves;
//         the 16-byte reads of rows 2g, 2g + 1 by one 16-lane group do as well.
//   bf16: one 32-row x 64-column strip at a time, row pitch 128 B.  Every lane rounds its two rows of one
//         column into a dword, neighbouring lanes exchange it (DPP quad permute) and a byte permute leaves
//         the even lane with columns (c, c + 1) of row R and the odd lane with columns (c - 1, c) of
//         row R + 1, packed into one dword; the 64-byte half of the row that
//         block j goes to is j ^ ((R >> 2) & 1), for the same bank reason.
// Compile-time indices throughout: the accumulators must never be indexed dynamically (they would
// move to scratch memory).  Edge tiles and result pitches that are not a multiple of 16 bytes take
// the guarded element-wise path.
//
// LOADS_FIRST (persistent kernel): direct-to-LDS loads of the next tile are in flight when the
// epilogue starts, and the caller wants to run its next two reduction steps while the stores of this
// tile drain.  Loads and stores share one in-order completion counter, and once a store is pending
// behind a load the compiler no longer trusts any count on it and falls back to "wait for
// everything" at the next LDS read.  So here (a) the in-flight loads are waited for right before the
// first store, when the first block is already staged and they are about a microsecond old, and (b)
// the stores are issued as inline assembly, outside the compiler's bookkeeping; every later wait on
// the counter is an explicit one that counts them in (see the tile loop of the persistent kernel).
__global__ __launch_bounds__(256) void fill_rowmax_kernel(GemmPlan p) {
    const GemmShard& s = p.s[blockIdx.y];
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < s.m) s.rowmax[r] = -__builtin_inff();
}


template <int BM, int BN, int TM, int TN, int FM, int FN, int EPI, typename OutT, bool LOADS_FIRST = false>
__device__ __attribute__((always_inline)) inline void store_tile(const f32x16 (&acc)[FM][FN], const GemmShard& s, int m0, int n0, int wm, int wn, int lane, char* stage) {
    OutT* C = static_cast<OutT*>(s.c);
    constexpr int EPV = 16 / (int)sizeof(OutT);   // elements per 16-byte store
    const bool whole = m0 + BM <= s.m && n0 + BN <= s.n && s.ldc % EPV == 0;
    [[maybe_unused]] const bool stream = (s.ldc * (int)sizeof(OutT)) % 128 == 0;
    if (whole) {
        const int wave = (int)(threadIdx.x >> 6);
        const int h = lane >> 5, c = lane & 31;
        // lane parts of the LDS offsets, opaque so that every address is object + (lane part + constant)
        int rd = wave * STAGE_BYTES + (((lane >> 3) ^ h) * 128) + (lane & 7) * 16;
        if constexpr (sizeof(OutT) == 2) rd = wave * STAGE_BYTES + (lane >> 3) * 128 + (((lane & 7) * 16) ^ (64 * h));
        asm volatile("" : "+v"(rd));
        OutT* cg = C + (int64_t)(m0 + wm * TM + (lane >> 3)) * s.ldc + (n0 + wn * TN + (lane & 7) * EPV);
        if constexpr (sizeof(OutT) == 4) {
            int w0 = wave * STAGE_BYTES + h * 640 + c * 4;   // rows with r % 4 even: (b ^ h) = b + h
            int w1 = wave * STAGE_BYTES + h * 384 + c * 4;   // rows with r % 4 odd:  (b ^ h) = b - h
            asm volatile("" : "+v"(w0));
            asm volatile("" : "+v"(w1));
            static_for<FM * FN>([&](auto idx) {
                constexpr int i = decltype(idx)::value / FN, j = decltype(idx)::value % FN;
                static_for<16>([&](auto ridx) {
                    constexpr int r = decltype(ridx)::value;
                    constexpr int off = (8 * (r >> 2) + (r & 3)) * 128;
                    *reinterpret_cast<float*>(stage + (((r & 1) ? w1 : w0) + off)) = mfma_epilogue<EPI>(acc[i][j][r]);
                });
                __builtin_amdgcn_wave_barrier();
                static_for<4>([&](auto qidx) {
                    constexpr int q = decltype(qidx)::value;
                    const f32x4 v = *reinterpret_cast<const f32x4*>(stage + (rd + q * 1024));
                    f32x4* dst = reinterpret_cast<f32x4*>(cg + (int64_t)(i * 32 + q * 8) * s.ldc + j * 32);
                    if constexpr (LOADS_FIRST) {
                        if constexpr (decltype(idx)::value == 0 && q == 0) __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
                        store16_untracked(dst, v, stream);
                    } else {
                        __builtin_nontemporal_store(v, dst);
                    }
                });
                __builtin_amdgcn_wave_barrier();
            });
        } else {
            static_assert(FN % 2 == 0, "bf16 results are staged in strips of two 32-column blocks");
            const int odd = lane & 1;
            // even lane: row R, columns (c, c + 1) = low halves of (own, neighbour); odd lane: row R + 1, columns
            // (c - 1, c) = high halves of (neighbour, own).  Byte selectors: 0-3 own, 4-7 neighbour.
            const uint32_t pick = odd ? 0x03020706u : 0x05040100u;
            [[maybe_unused]] float rm[FM][4];   // EPI_ROWMAX: maxima of rows 32 i + 8 q + lane / 8 over this wave's columns
            if constexpr (EPI == EPI_ROWMAX) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) rm[i][q] = -__builtin_inff();
            }
            int w0 = wave * STAGE_BYTES + (4 * h + odd) * 128 + h * 64 + (c >> 1) * 4;         // block j even
            int w1 = wave * STAGE_BYTES + (4 * h + odd) * 128 + (1 - h) * 64 + (c >> 1) * 4;   // block j odd
            asm volatile("" : "+v"(w0));
            asm volatile("" : "+v"(w1));
            static_for<FM * (FN / 2)>([&](auto idx) {
                constexpr int i = decltype(idx)::value / (FN / 2), jp = decltype(idx)::value % (FN / 2);
                static_for<2>([&](auto jidx) {
                    constexpr int j = 2 * jp + decltype(jidx)::value;
                    static_for<8>([&](auto pidx) {
                        constexpr int r = 2 * decltype(pidx)::value;             // rows R (r) and R + 1 (r + 1)
                        // own column, rows R and R + 1, rounded; then one byte permute with the neighbour's pair
                        const uint32_t own = f32_to_bf16x2(mfma_epilogue<EPI>(acc[i][j][r]), mfma_epilogue<EPI>(acc[i][j][r + 1]));
                        const uint32_t nb = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
                        const uint32_t packed = __builtin_amdgcn_perm(nb, own, pick);
                        constexpr int off = (8 * (r >> 2) + (r & 3)) * 128;
                        *reinterpret_cast<uint32_t*>(stage + (((j & 1) ? w1 : w0) + off)) = packed;
                    });
                });
                __builtin_amdgcn_wave_barrier();
                static_for<4>([&](auto qidx) {
                    constexpr int q = decltype(qidx)::value;
                    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + (rd + q * 1024));
                    u32x4* dst = reinterpret_cast<u32x4*>(cg + (int64_t)(i * 32 + q * 8) * s.ldc + jp * 64);
                    if constexpr (EPI == EPI_ROWMAX) {
                        // this lane's 8 stored values, then the 8 lanes that share the row (quads, then
                        // the two quads of the group through the half-row mirror)
                        float mx = fmaxf(__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xFFFF0000u));
#pragma unroll
                        for (int d = 1; d < 4; ++d) mx = fmaxf(mx, fmaxf(__uint_as_float(v[d] << 16), __uint_as_float(v[d] & 0xFFFF0000u)));
                        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0xB1, 0xF, 0xF, false)));    // quad_perm [1,0,3,2]
                        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0x4E, 0xF, 0xF, false)));    // quad_perm [2,3,0,1]
                        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0x141, 0xF, 0xF, false)));   // row_half_mirror
                        rm[i][q] = fmaxf(rm[i][q], mx);
                    }
                    if constexpr (LOADS_FIRST) {
                        if constexpr (decltype(idx)::value == 0 && q == 0) __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
                        store16_untracked(dst, v, stream);
                    } else {
                        __builtin_nontemporal_store(v, dst);
                    }
                });
                __builtin_amdgcn_wave_barrier();
            });
            if constexpr (EPI == EPI_ROWMAX) {
                // The WN waves of one wave row hold maxima of the same TM rows over different columns:
                // publish them in the (now idle) windows, one workgroup barrier, then the first wave
                // of every wave row combines them and issues one atomic per row (a quarter of the
                // atomics a wave-by-wave update would need).  The windows are next written in the
                // next tile's epilogue, several barriers of the reduction loop later.
                constexpr int WN_ = BN / TN;
                float* win = reinterpret_cast<float*>(stage + wave * STAGE_BYTES);
                if ((lane & 7) == 0) {
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q) win[i * 32 + q * 8 + (lane >> 3)] = rm[i][q];
                }
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                if (wn == 0) {
#pragma unroll
                    for (int t = 0; t < TM / 64; ++t) {
                        const int row = lane + 64 * t;
                        float mx = win[row];
#pragma unroll
                        for (int w = 1; w < WN_; ++w) mx = fmaxf(mx, reinterpret_cast<const float*>(stage + (wave + w) * STAGE_BYTES)[row]);
                        atomic_max_f32_untracked(s.rowmax + (m0 + wm * TM + row), mx);
                    }
                }
            }
        }
        return;
    }
    const int cn = lane & 31, rm = 4 * (lane >> 5);
    static_for<FM * FN>([&](auto idx) {
        constexpr int i = decltype(idx)::value / FN, j = decltype(idx)::value % FN;
        const int n = n0 + wn * TN + j * 32 + cn;
        const int mb = m0 + wm * TM + i * 32 + rm;
        OutT* cp = C + (int64_t)mb * s.ldc + n;
        static_for<16>([&](auto ridx) {
            constexpr int r = decltype(ridx)::value;
            const int m = mb + 8 * (r >> 2) + (r & 3);
            const float v = mfma_epilogue<EPI>(acc[i][j][r]);
            if (m < s.m && n < s.n) {
                if constexpr (LOADS_FIRST) store_out_untracked(cp, (int64_t)(8 * (r >> 2) + (r & 3)) * s.ldc, v);
                else store_out(cp, (int64_t)(8 * (r >> 2) + (r & 3)) * s.ldc, v);
                if constexpr (EPI == EPI_ROWMAX) atomic_max_f32_untracked(s.rowmax + m, bf16_to_f32(f32_to_bf16(v)));
            }
        });
    });
    if constexpr (LOADS_FIRST) __builtin_amdgcn_s_waitcnt(vmcnt_only(0));   // edge tile: loads and stores alike
}

// Epilogue for accumulators of v_mfma_f32_16x16x32_bf16 (persistent kernel): every 16 x 16 block holds
// D[4 (lane / 16) + r][lane % 16] = acc[r], r = 0..3.  Same per-wave 4 KB window, same read side (each lane
// ends up with 16 consecutive bytes of a row; eight 128-byte row segments per store instruction) and the
// same global addressing as store_tile; only the way the accumulators enter the window differs.
//   fp32: a 32 x 32 region (2 x 2 blocks) at a time, row pitch 128 B.  One write instruction covers rows
//         4 g + r for g = lane / 16 = 0..3, 16 dwords each: row R is kept at R ^ ((R >> 2) & 1) and its
//         two 64-byte halves are swapped when (R >> 3) & 1, which puts the four rows on 4 x 16 banks.
//   bf16: a 32-row x 64-column strip (2 x 4 blocks) at a time.  Lanes round and pair their rows R, R + 1
//         and exchange with the neighbouring column as in store_tile; one write instruction covers rows
//         4 g + (lane & 1), 8 dwords each: the 32-byte column group j is kept at j ^ g.
template <int BM, int BN, int TM, int TN, int EPI, typename OutT>
__device__ __attribute__((always_inline)) inline void store_tile16(const f32x4 (&acc)[TM / 16][TN / 16], const GemmShard& s, int m0, int n0, int wm, int wn, int lane, char* stage) {
    constexpr int FM = TM / 32, FN = TN / 32;       // 32 x 32 regions, as in store_tile
    OutT* C = static_cast<OutT*>(s.c);
    constexpr int EPV = 16 / (int)sizeof(OutT);
    const bool whole = m0 + BM <= s.m && n0 + BN <= s.n && s.ldc % EPV == 0;
    [[maybe_unused]] const bool stream = (s.ldc * (int)sizeof(OutT)) % 128 == 0;
    // Every lane constant of the epilogue is derived from this copy of the lane id, which the compiler cannot
    // move out of the tile loop: they are recomputed per tile (a few dozen instructions) instead of occupying
    // registers all through the reduction loop, which has none to spare.
    asm volatile("" : "+v"(lane));
    const int g = lane >> 4, c = lane & 15;
    if (whole) {
        const int wave = (int)(threadIdx.x >> 6);
        const int h = lane >> 5;
        OutT* cg = C + (int64_t)(m0 + wm * TM + (lane >> 3)) * s.ldc + (n0 + wn * TN + (lane & 7) * EPV);
        if constexpr (sizeof(OutT) == 4) {
            // read side: logical row (lane / 8) + 8 q, logical 16-byte chunk lane % 8
            int rd0 = wave * STAGE_BYTES + (((lane >> 3) ^ h) * 128) + (lane & 7) * 16;            // q even
            int rd1 = wave * STAGE_BYTES + (((lane >> 3) ^ h) * 128) + (((lane & 7) ^ 4) * 16);      // q odd: halves swapped
            asm volatile("" : "+v"(rd0));
            asm volatile("" : "+v"(rd1));
            // write side: [r parity][jb]
            int w[2][2];
#pragma unroll
            for (int rp = 0; rp < 2; ++rp)
#pragma unroll
                for (int jb = 0; jb < 2; ++jb) {
                    w[rp][jb] = wave * STAGE_BYTES + (4 * g + (rp ^ (g & 1))) * 128 + (16 * (jb ^ (g >> 1)) + c) * 4;
                    asm volatile("" : "+v"(w[rp][jb]));
                }
            static_for<FM * FN>([&](auto idx) {
                constexpr int i = decltype(idx)::value / FN, j = decltype(idx)::value % FN;
                static_for<2>([&](auto ibx) {
                    constexpr int ib = decltype(ibx)::value;
                    static_for<2>([&](auto jbx) {
                        constexpr int jb = decltype(jbx)::value;
                        static_for<4>([&](auto ridx) {
                            constexpr int r = decltype(ridx)::value;
                            constexpr int off = (16 * ib + (r & 2)) * 128;
                            *reinterpret_cast<float*>(stage + (w[r & 1][jb] + off)) = mfma_epilogue<EPI>(acc[2 * i + ib][2 * j + jb][r]);
                        });
                    });
                });
                __builtin_amdgcn_wave_barrier();
                static_for<4>([&](auto qidx) {
                    constexpr int q = decltype(qidx)::value;
                    const f32x4 v = *reinterpret_cast<const f32x4*>(stage + (((q & 1) ? rd1 : rd0) + q * 1024));
                    f32x4* dst = reinterpret_cast<f32x4*>(cg + (int64_t)(i * 32 + q * 8) * s.ldc + j * 32);
                    if constexpr (decltype(idx)::value == 0 && q == 0) __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
                    store16_untracked(dst, v, stream);
                });
                __builtin_amdgcn_wave_barrier();
            });
        } else {
            static_assert(TN == 64, "bf16 results are staged in strips of 64 columns");
            const int odd = lane & 1;
            const uint32_t pick = odd ? 0x03020706u : 0x05040100u;
            [[maybe_unused]] float rm[FM][4];
            if constexpr (EPI == EPI_ROWMAX) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) rm[i][q] = -__builtin_inff();
            }
            // read side: logical row (lane / 8) + 8 q, chunk lane % 8; the row's column groups are kept at j ^ g(row)
            int rd0 = wave * STAGE_BYTES + (lane >> 3) * 128 + (((lane & 7) ^ (2 * h)) * 16);           // q even: g(row) = h
            int rd1 = wave * STAGE_BYTES + (lane >> 3) * 128 + (((lane & 7) ^ (2 * h + 4)) * 16);       // q odd:  g(row) = h + 2
            asm volatile("" : "+v"(rd0));
            asm volatile("" : "+v"(rd1));
            int w[4];   // [j]
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                w[j] = wave * STAGE_BYTES + (4 * g + odd) * 128 + ((((j ^ g) << 3) + (c >> 1)) * 4);
                asm volatile("" : "+v"(w[j]));
            }
            static_for<FM>([&](auto idx) {
                constexpr int i = decltype(idx)::value;
                static_for<2>([&](auto ibx) {
                    constexpr int ib = decltype(ibx)::value;
                    static_for<4>([&](auto jidx) {
                        constexpr int j = decltype(jidx)::value;
                        static_for<2>([&](auto pidx) {
                            constexpr int r = 2 * decltype(pidx)::value;
                            const uint32_t own = f32_to_bf16x2(mfma_epilogue<EPI>(acc[2 * i + ib][j][r]), mfma_epilogue<EPI>(acc[2 * i + ib][j][r + 1]));
                            const uint32_t nb = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
                            const uint32_t packed = __builtin_amdgcn_perm(nb, own, pick);
                            constexpr int off = (16 * ib + r) * 128;
                            *reinterpret_cast<uint32_t*>(stage + (w[j] + off)) = packed;
                        });
                    });
                });
                __builtin_amdgcn_wave_barrier();
                static_for<4>([&](auto qidx) {
                    constexpr int q = decltype(qidx)::value;
                    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + (((q & 1) ? rd1 : rd0) + q * 1024));
                    u32x4* dst = reinterpret_cast<u32x4*>(cg + (int64_t)(i * 32 + q * 8) * s.ldc);
                    if constexpr (EPI == EPI_ROWMAX) {
                        float mx = fmaxf(__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xFFFF0000u));
#pragma unroll
                        for (int d = 1; d < 4; ++d) mx = fmaxf(mx, fmaxf(__uint_as_float(v[d] << 16), __uint_as_float(v[d] & 0xFFFF0000u)));
                        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0xB1, 0xF, 0xF, false)));
                        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0x4E, 0xF, 0xF, false)));
                        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0x141, 0xF, 0xF, false)));
                        rm[i][q] = fmaxf(rm[i][q], mx);
                    }
                    if constexpr (decltype(idx)::value == 0 && q == 0) __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
                    store16_untracked(dst, v, stream);
                });
                __builtin_amdgcn_wave_barrier();
            });
            if constexpr (EPI == EPI_ROWMAX) {
                constexpr int WN_ = BN / TN;
                float* win = reinterpret_cast<float*>(stage + wave * STAGE_BYTES);
                if ((lane & 7) == 0) {
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q) win[i * 32 + q * 8 + (lane >> 3)] = rm[i][q];
                }
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                if (wn == 0) {
#pragma unroll
                    for (int t = 0; t < TM / 64; ++t) {
                        const int row = lane + 64 * t;
                        float mx = win[row];
#pragma unroll
                        for (int ww = 1; ww < WN_; ++ww) mx = fmaxf(mx, reinterpret_cast<const float*>(stage + (wave + ww) * STAGE_BYTES)[row]);
                        atomic_max_f32_untracked(s.rowmax + (m0 + wm * TM + row), mx);
                    }
                }
            }
        }
        return;
    }
    // edge tiles: element by element, guarded
    static_for<(TM / 16) * (TN / 16)>([&](auto idx) {
        constexpr int i = decltype(idx)::value / (TN / 16), j = decltype(idx)::value % (TN / 16);
        const int n = n0 + wn * TN + j * 16 + c;
        const int mb = m0 + wm * TM + i * 16 + 4 * g;
        OutT* cp = C + (int64_t)mb * s.ldc + n;
        static_for<4>([&](auto ridx) {
            constexpr int r = decltype(ridx)::value;
            const int m = mb + r;
            const float v = mfma_epilogue<EPI>(acc[i][j][r]);
            if (m < s.m && n < s.n) {
                store_out_untracked(cp, (int64_t)r * s.ldc, v);
                if constexpr (EPI == EPI_ROWMAX) atomic_max_f32_untracked(s.rowmax + m, bf16_to_f32(f32_to_bf16(v)));
            }
        });
    });
    __builtin_amdgcn_s_waitcnt(vmcnt_only(0));   // edge tile: loads and stores alike
}

// Scheduling hint for one phase of NMFMA matrix instructions: let one LDS read and (for the first NVM
// of them) one global->LDS load issue behind each MFMA, so that the operands of the NEXT phase stream
// in underneath the matrix pipe instead of in a burst right before they are needed.
template <int NMFMA, int NDS, int NVM>
__device__ inline void pace() {
    static_for<NMFMA>([&](auto i) {
        constexpr int I = decltype(i)::value;
        constexpr int nds = NDS * (I + 1) / NMFMA - NDS * I / NMFMA;   // spread evenly, all before the phase ends
        constexpr int nvm = NVM * (I + 1) / NMFMA - NVM * I / NMFMA;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // 1 MFMA
        if constexpr (nds > 0) __builtin_amdgcn_sched_group_barrier(0x100, nds, 0);   // LDS reads
        if constexpr (nvm > 0) __builtin_amdgcn_sched_group_barrier(0x010, nvm, 0);   // VMEM
    });
}

// Schedule of one reduction step t (LDS stage t & 1 holds tile t):
//   phase 0..2: issue the direct-to-LDS loads of tile t + 1 into the other stage (phase 0 only;
//               that stage was last read in step t - 1), read the fragments of ks + 1, run the
//               MFMAs of ks
//   wait for this wave's loads, workgroup barrier      (tile t + 1 complete, stage t & 1 free)
//   phase 3:    read the fragments of (t + 1, ks = 0) underneath the MFMAs of (t, ks = 3)
// The four stages are separate __shared__ objects on purpose: the compiler then knows that a
// direct-to-LDS load into one stage cannot alias the fragment reads of the other and does not
// serialise them with a vmcnt wait.
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int ODD, int EPI, typename OutT>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(GemmPlan p, int tm, int tn, int order) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;   // wave tile
    constexpr int FM = TM / 32, FN = TN / 32;   // 32x32 MFMA tiles per wave
    constexpr int NDS = (A_KC ? FM : 2 * FM) + (B_KC ? FN : 2 * FN);   // LDS reads per phase
    using TA = Tile<BM, A_KC, NT>;
    using TB = Tile<BN, B_KC, NT>;
    constexpr int NVM = TA::PER_THREAD + TB::PER_THREAD;                // loads per step
    __shared__ __attribute__((aligned(1024))) char sA0[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA1[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB0[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB1[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sOut[WM * WN * STAGE_BYTES];   // epilogue windows, one per wave

    const TileCoord tc = map_tile(blockIdx.x, gridDim.x, tm, tn, p.groups, order);
    if (!tc.valid) return;
    const GemmShard s = p.s[tc.g];
    const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
    if (m0 >= s.m || n0 >= s.n) return;   // uneven shards: this one has fewer tiles

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    gbl_char* A = (gbl_char*)s.a;
    gbl_char* B = (gbl_char*)s.b;

    uint32_t offa[TA::PER_THREAD], offb[TB::PER_THREAD];
#pragma unroll
    for (int it = 0; it < TA::PER_THREAD; ++it) offa[it] = TA::src_offset(s.lda, m0, s.m, it * NT + tid);
#pragma unroll
    for (int it = 0; it < TB::PER_THREAD; ++it) offb[it] = TB::src_offset(s.ldb, n0, s.n, it * NT + tid);
    const uint32_t stepa = TA::step_bytes(s.lda), stepb = TB::step_bytes(s.ldb);

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    bf16x8 fa[2][FM], fb[2][FN];
    int loa[TA::template nlo<FM>()], lob[TB::template nlo<FN>()];
#pragma unroll
    for (int x = 0; x < TA::template nlo<FM>(); ++x) loa[x] = TA::lane_offset(x, wm * TM, lane);
#pragma unroll
    for (int x = 0; x < TB::template nlo<FN>(); ++x) lob[x] = TB::lane_offset(x, wn * TN, lane);

    auto read_frags = [&](const char* sa, const char* sb, int ks, int slot) {
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[slot][j] = TB::frag(sb, lob, j, ks);
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[slot][i] = TA::frag(sa, loa, i, ks);
    };
    auto mfmas = [&](int slot) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
    };
    // One reduction step computing from stage CUR.  It is branch-free so that the whole step is one
    // scheduling region: the loads of the next tile are ALWAYS issued (after the last tile the source
    // simply stops advancing, so the reload stays in bounds and nobody reads it) and the fragments of
    // the next stage are always read.
    const int steps = s.kk / BK;
    int t = 0;
    auto step = [&](auto cur) {
        constexpr int CUR = decltype(cur)::value;
        const char* sa = CUR ? sA1 : sA0;
        const char* sb = CUR ? sB1 : sB0;
        char* da = CUR ? sA0 : sA1;
        char* db = CUR ? sB0 : sB1;
        TA::load_direct(da, A, offa, wave);
        TB::load_direct(db, B, offb, wave);
        ++t;
        const bool adv = t + 1 < steps;      // tile t + 1 exists (t already counts this step)
        A += adv ? stepa : 0u;
        B += adv ? stepb : 0u;
        read_frags(sa, sb, 1, 1);
        mfmas(0);
        pace<FM * FN, NDS, NVM>();
        read_frags(sa, sb, 2, 0);
        mfmas(1);
        pace<FM * FN, NDS, 0>();
        read_frags(sa, sb, 3, 1);
        mfmas(0);
        pace<FM * FN, NDS, 0>();
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0): loads landed, fragment reads returned
        __builtin_amdgcn_s_barrier();
        read_frags(da, db, 0, 0);
        mfmas(1);
        pace<FM * FN, NDS, 0>();
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    TA::load_direct(sA0, A, offa, wave);
    TB::load_direct(sB0, B, offb, wave);
    __builtin_amdgcn_s_waitcnt(0x0070);
    if (steps > 1) {
        A += stepa;
        B += stepb;
    }
    __builtin_amdgcn_s_barrier();
    read_frags(sA0, sB0, 0, 0);
    for (int pair = 0; pair < steps / 2; ++pair) {
        step(I0{});
        step(I1{});
    }
    if (steps & 1) step(I0{});

    store_tile<BM, BN, TM, TN, FM, FN, EPI, OutT>(acc, s, m0, n0, wm, wn, lane, sOut);
}

// ------------------------------------------------------------------------------------------------
// Deeper pipeline: NST LDS stages of 32 reduction elements each (same 128 KB as 2 x 64 when
// NST = 4), so that NST - 1 tiles are in flight while one is being multiplied.  One step t:
//   issue the loads of tile t + NST - 1 into the stage that step t - 1 just finished with
//   read the fragments of (t, ks = 1), run the MFMAs of (t, ks = 0)
//   wait until only the loads of tiles t + 2 .. are outstanding (they complete in order), barrier
//   read the fragments of (t + 1, ks = 0), run the MFMAs of (t, ks = 1)
// ------------------------------------------------------------------------------------------------
// Tiles of at most 256 x 128 on 4 waves are built to run TWO workgroups per CU (<= 256 registers per
// lane, <= 80 KB LDS): while one stores its results the other keeps the matrix cores busy.
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int NST, int EPI, typename OutT>
__global__ __launch_bounds__(WM * WN * 64, (BM * BN <= 256 * 128 && WM * WN == 4) ? 2 : 1) void gemm_mfma_pipe_kernel(GemmPlan p, int tm, int tn, int order) {
    constexpr int BKT = 32;
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int NDS = (A_KC ? FM : 2 * FM) + (B_KC ? FN : 2 * FN);
    using TA = Tile<BM, A_KC, NT, BKT>;
    using TB = Tile<BN, B_KC, NT, BKT>;
    constexpr int NVM = TA::PER_THREAD + TB::PER_THREAD;
    static_assert(NST >= 3 && NST <= 5, "3 to 5 stages");
    static_assert((NST - 2) * NVM < 64, "vmcnt field");
    __shared__ __attribute__((aligned(1024))) char sA0[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA1[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA2[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA3[NST > 3 ? TA::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sA4[NST > 4 ? TA::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sB0[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB1[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB2[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB3[NST > 3 ? TB::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sB4[NST > 4 ? TB::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sOut[WM * WN * STAGE_BYTES];   // epilogue windows, one per wave
    auto stA = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sA0; else if constexpr (I == 1) return sA1; else if constexpr (I == 2) return sA2;
        else if constexpr (I == 3) return sA3; else return sA4;
    };
    auto stB = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sB0; else if constexpr (I == 1) return sB1; else if constexpr (I == 2) return sB2;
        else if constexpr (I == 3) return sB3; else return sB4;
    };

    const TileCoord tc = map_tile(blockIdx.x, gridDim.x, tm, tn, p.groups, order);
    if (!tc.valid) return;
    const GemmShard s = p.s[tc.g];
    const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
    if (m0 >= s.m || n0 >= s.n) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    gbl_char* A = (gbl_char*)s.a;
    gbl_char* B = (gbl_char*)s.b;

    uint32_t offa[TA::PER_THREAD], offb[TB::PER_THREAD];
#pragma unroll
    for (int it = 0; it < TA::PER_THREAD; ++it) offa[it] = TA::src_offset(s.lda, m0, s.m, it * NT + tid);
#pragma unroll
    for (int it = 0; it < TB::PER_THREAD; ++it) offb[it] = TB::src_offset(s.ldb, n0, s.n, it * NT + tid);
    const uint32_t stepa = TA::step_bytes(s.lda), stepb = TB::step_bytes(s.ldb);

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    bf16x8 fa[2][FM], fb[2][FN];
    int loa[TA::template nlo<FM>()], lob[TB::template nlo<FN>()];
#pragma unroll
    for (int x = 0; x < TA::template nlo<FM>(); ++x) loa[x] = TA::lane_offset(x, wm * TM, lane);
#pragma unroll
    for (int x = 0; x < TB::template nlo<FN>(); ++x) lob[x] = TB::lane_offset(x, wn * TN, lane);

    auto read_frags = [&](const char* sa, const char* sb, int ks, int slot) {
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[slot][j] = TB::frag(sb, lob, j, ks);
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[slot][i] = TA::frag(sa, loa, i, ks);
    };
    auto mfmas = [&](int slot) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
    };

    const int steps = s.kk / BKT;
    int loaded = 0;   // tiles whose loads have been issued; the source pointers sit on tile min(loaded, steps - 1)
    auto issue = [&](char* da, char* db) {
        TA::load_direct(da, A, offa, wave);
        TB::load_direct(db, B, offb, wave);
        ++loaded;
        const bool adv = loaded < steps;   // past the last tile the pointer stays: reloads are in bounds, unread
        A += adv ? stepa : 0u;
        B += adv ? stepb : 0u;
    };
    // s_waitcnt immediate: vmcnt(n), n < 64, split over bits 3:0 and 15:14; expcnt left at "no wait"
    constexpr int WAIT_KEEP = (NST - 2) * NVM;
    constexpr int WAIT_IMM = (WAIT_KEEP & 15) | ((WAIT_KEEP >> 4) << 14) | 0x0070;   // ... and lgkmcnt(0)

    auto step = [&](auto cur) {
        constexpr int CUR = decltype(cur)::value;
        using Nxt = std::integral_constant<int, (CUR + 1) % NST>;
        using Dst = std::integral_constant<int, (CUR + NST - 1) % NST>;
        issue(stA(Dst{}), stB(Dst{}));
        read_frags(stA(cur), stB(cur), 1, 1);
        mfmas(0);
        pace<FM * FN, NDS, NVM>();
        // This wave's part of the next tile has landed (later tiles may still fly) and its own
        // fragment reads have returned; then a bare hardware barrier.  __syncthreads() is not used:
        // its workgroup fence counts direct-to-LDS loads as LDS stores and would drain ALL of them.
        __builtin_amdgcn_s_waitcnt(WAIT_IMM);
        __builtin_amdgcn_s_barrier();
        read_frags(stA(Nxt{}), stB(Nxt{}), 0, 0);
        mfmas(1);
        pace<FM * FN, NDS, 0>();
    };

    static_for<NST - 1>([&](auto i) { issue(stA(i), stB(i)); });
    __builtin_amdgcn_s_waitcnt(WAIT_IMM);
    __builtin_amdgcn_s_barrier();
    read_frags(sA0, sB0, 0, 0);
    int t = 0;
    for (; t + NST <= steps; t += NST) static_for<NST>([&](auto i) { step(i); });
    const int rem = steps - t;   // 0 .. NST - 1 steps left, stage numbering continues from 0
    static_for<NST - 1>([&](auto i) {
        if (decltype(i)::value < rem) step(i);
    });
    __builtin_amdgcn_s_waitcnt(0x0070);   // drain the (unread) trailing loads before LDS is released

    store_tile<BM, BN, TM, TN, FM, FN, EPI, OutT>(acc, s, m0, n0, wm, wn, lane, sOut);
}

// The pipelined kernel on v_mfma_f32_16x16x32_bf16 (four stages; fragments, step and epilogue as in
// gemm_mfma_persist16_kernel): shapes whose reduction length is a multiple of 32 but not of 128.
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int NST, int EPI, typename OutT>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_pipe16_kernel(GemmPlan p, int tm, int tn, int order) {
    constexpr int BKT = 32;
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 16, FN = TN / 16;       // 16 x 16 blocks per wave
    static_assert(FM % 2 == 0, "the row blocks are multiplied in two halves");
    constexpr int HM = FM / 2;
    constexpr int NDS_A = A_KC ? HM : 2 * HM;
    constexpr int NDS_B = B_KC ? FN : 2 * FN;
    using TA = Tile<BM, A_KC, NT, BKT, true>;
    using TB = Tile<BN, B_KC, NT, BKT, true>;
    constexpr int NVM = TA::PER_THREAD + TB::PER_THREAD;
    static_assert(NST == 4, "the B fragments alternate between two slots by stage parity");
    static_assert((NST - 2) * NVM < 64, "vmcnt field");
    __shared__ __attribute__((aligned(1024))) char sA0[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA1[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA2[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA3[NST > 3 ? TA::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sA4[NST > 4 ? TA::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sB0[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB1[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB2[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB3[NST > 3 ? TB::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sB4[NST > 4 ? TB::BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char sOut[WM * WN * STAGE_BYTES];   // epilogue windows, one per wave
    auto stA = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sA0; else if constexpr (I == 1) return sA1; else if constexpr (I == 2) return sA2;
        else if constexpr (I == 3) return sA3; else return sA4;
    };
    auto stB = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sB0; else if constexpr (I == 1) return sB1; else if constexpr (I == 2) return sB2;
        else if constexpr (I == 3) return sB3; else return sB4;
    };

    const TileCoord tc = map_tile(blockIdx.x, gridDim.x, tm, tn, p.groups, order);
    if (!tc.valid) return;
    const GemmShard s = p.s[tc.g];
    const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
    if (m0 >= s.m || n0 >= s.n) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    gbl_char* A = (gbl_char*)s.a;
    gbl_char* B = (gbl_char*)s.b;

    uint32_t offa[TA::PER_THREAD], offb[TB::PER_THREAD];
#pragma unroll
    for (int it = 0; it < TA::PER_THREAD; ++it) offa[it] = TA::src_offset(s.lda, m0, s.m, it * NT + tid);
#pragma unroll
    for (int it = 0; it < TB::PER_THREAD; ++it) offb[it] = TB::src_offset(s.ldb, n0, s.n, it * NT + tid);
    const uint32_t stepa = TA::step_bytes(s.lda), stepb = TB::step_bytes(s.ldb);

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

    bf16x8 fa[2][HM], fb[2][FN];
    static_assert((A_KC || (TM % 64 == 0 && FM <= 8)) && (B_KC || (TN % 64 == 0 && FN <= 4)), "see Tile::lane_offset16");
    const int loa = TA::lane_offset16(wm * TM, lane), lob = TB::lane_offset16(wn * TN, lane);
    auto read_a = [&](const char* sa, int half) {
#pragma unroll
        for (int i = 0; i < HM; ++i) fa[half][i] = TA::frag16(sa, loa, half * HM + i);
    };
    auto read_b = [&](const char* sb, int slot) {
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[slot][j] = TB::frag16(sb, lob, j);
    };
    auto mfmas = [&](int half, int slot) {
#pragma unroll
        for (int i = 0; i < HM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[half * HM + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[half][i], fb[slot][j], acc[half * HM + i][j], 0, 0, 0);
    };

    const int steps = s.kk / BKT;
    int loaded = 0;   // tiles whose loads have been issued; the source pointers sit on tile min(loaded, steps - 1)
    auto issue = [&](char* da, char* db) {
        TA::load_direct(da, A, offa, wave);
        TB::load_direct(db, B, offb, wave);
        ++loaded;
        const bool adv = loaded < steps;   // past the last tile the pointer stays: reloads are in bounds, unread
        A += adv ? stepa : 0u;
        B += adv ? stepb : 0u;
    };
    // s_waitcnt immediate: vmcnt(n), n < 64, split over bits 3:0 and 15:14; expcnt left at "no wait"
    constexpr int WAIT_KEEP = (NST - 2) * NVM;
    constexpr int WAIT_IMM = (WAIT_KEEP & 15) | ((WAIT_KEEP >> 4) << 14) | 0x0070;   // ... and lgkmcnt(0)

    auto step = [&](auto cur) {
        constexpr int CUR = decltype(cur)::value;
        using Nxt = std::integral_constant<int, (CUR + 1) % NST>;
        using Dst = std::integral_constant<int, (CUR + NST - 1) % NST>;
        issue(stA(Dst{}), stB(Dst{}));
        read_a(stA(cur), 1);
        mfmas(0, CUR & 1);
        pace<HM * FN, NDS_A, NVM>();
        // This wave's part of the next tile has landed (later tiles may still fly) and its own
        // fragment reads have returned; then a bare hardware barrier.  __syncthreads() is not used:
        // its workgroup fence counts direct-to-LDS loads as LDS stores and would drain ALL of them.
        __builtin_amdgcn_s_waitcnt(WAIT_IMM);
        __builtin_amdgcn_s_barrier();
        read_a(stA(Nxt{}), 0);
        read_b(stB(Nxt{}), (CUR + 1) & 1);
        mfmas(1, CUR & 1);
        pace<HM * FN, NDS_A + NDS_B, 0>();
    };

    static_for<NST - 1>([&](auto i) { issue(stA(i), stB(i)); });
    __builtin_amdgcn_s_waitcnt(WAIT_IMM);
    __builtin_amdgcn_s_barrier();
    read_a(sA0, 0);
    read_b(sB0, 0);
    int t = 0;
    for (; t + NST <= steps; t += NST) static_for<NST>([&](auto i) { step(i); });
    const int rem = steps - t;   // 0 .. NST - 1 steps left, stage numbering continues from 0
    static_for<NST - 1>([&](auto i) {
        if (decltype(i)::value < rem) step(i);
    });
    __builtin_amdgcn_s_waitcnt(0x0070);   // drain the (unread) trailing loads before LDS is released

    store_tile16<BM, BN, TM, TN, EPI, OutT>(acc, s, m0, n0, wm, wn, lane, sOut);
}

// ------------------------------------------------------------------------------------------------
// Persistent form of the pipelined kernel: one workgroup per CU walks its tiles v = b, b + G, ...
// (G = grid size, a multiple of 8, so a workgroup stays on the XCD the tile walk assigns) and the
// load stream never drains: the loads for the first stages of tile i + 1 are issued during the last
// steps of tile i, so neither the prologue latency nor the workgroup turn-around (a new workgroup
// cannot start before the old one's stores have drained) nor the output stores themselves stop the
// matrix pipe for longer than it takes to ISSUE the stores.
//
// Memory-counter bookkeeping (loads and stores complete in issue order on one counter; every wait in
// this kernel is explicit, its loads and stores being issued outside the compiler's own accounting):
//   * a normal step issues the loads of the stage three ahead, then waits until at most the two
//     youngest stages are outstanding, which means the stage it reads next has landed;
//   * the epilogue waits for everything once, right before its first store, when the only things in
//     flight are the next tile's stages 1 and 2, issued one and two steps earlier;
//   * the first two steps of the next tile therefore need no wait at all, and the stores drain
//     underneath them; the third step's "all but the two youngest stages" covers the stores too.
// Requires every shard's reduction extent to be a multiple of 32 NST.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int NST, int EPI, typename OutT>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_persist_kernel(GemmPlan p, int tm, int tn, int order, int nblk) {
    constexpr int BKT = 32;
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int NDS = (A_KC ? FM : 2 * FM) + (B_KC ? FN : 2 * FN);
    using TA = Tile<BM, A_KC, NT, BKT>;
    using TB = Tile<BN, B_KC, NT, BKT>;
    constexpr int NVM = TA::PER_THREAD + TB::PER_THREAD;
    constexpr int WAIT_KEEP = (NST - 2) * NVM;
    static_assert(NST == 4, "written for four stages");
    __shared__ __attribute__((aligned(1024))) char sA0[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA1[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA2[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA3[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB0[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB1[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB2[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB3[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sOut[WM * WN * STAGE_BYTES];   // epilogue windows, one per wave
    auto stA = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sA0; else if constexpr (I == 1) return sA1; else if constexpr (I == 2) return sA2; else return sA3;
    };
    auto stB = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sB0; else if constexpr (I == 1) return sB1; else if constexpr (I == 2) return sB2; else return sB3;
    };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int G = gridDim.x;

    // first valid tile at or after virtual block v (uneven shards have fewer tiles than tm x tn)
    auto next_valid = [&](int v) {
        for (; v < nblk; v += G) {
            const TileCoord tc = map_tile(v, nblk, tm, tn, p.groups, order);
            if (tc.valid && tc.tile_m * BM < p.s[tc.g].m && tc.tile_n * BN < p.s[tc.g].n) break;
        }
        return v;
    };

    // ---- load cursor: always exactly NST - 1 stages ahead of the compute cursor ------------------
    gbl_char* A = nullptr;
    gbl_char* B = nullptr;
    uint32_t offa[TA::PER_THREAD], offb[TB::PER_THREAD];
    uint32_t stepa = 0, stepb = 0;
    const int first = next_valid(blockIdx.x);
    if (first >= nblk) return;         // nothing for this workgroup
    auto open_tile = [&](int v) {
        const TileCoord tc = map_tile(v, nblk, tm, tn, p.groups, order);
        const GemmShard& s = p.s[tc.g];
        A = (gbl_char*)s.a;
        B = (gbl_char*)s.b;
#pragma unroll
        for (int it = 0; it < TA::PER_THREAD; ++it) offa[it] = TA::src_offset(s.lda, tc.tile_m * BM, s.m, it * NT + tid);
#pragma unroll
        for (int it = 0; it < TB::PER_THREAD; ++it) offb[it] = TB::src_offset(s.ldb, tc.tile_n * BN, s.n, it * NT + tid);
        stepa = TA::step_bytes(s.lda);
        stepb = TB::step_bytes(s.ldb);
    };
    open_tile(first);
    // Branch-free: always NVM loads (the wait counts rely on it), then one stage forward.  Because a
    // tile has a multiple of NST stages, the cursor leaves a tile exactly after step 0 of the tile's
    // last round; the tile loop below re-opens it there.  Past the last tile the steps are zeroed, so
    // the last stage is simply re-read (in bounds, never used).
    auto issue = [&](char* da, char* db) {
        TA::load_direct_untracked(da, A, offa, wave);
        TB::load_direct_untracked(db, B, offb, wave);
        A += stepa;
        B += stepb;
    };

    // ---- compute side --------------------------------------------------------------------------
    f32x16 acc[FM][FN];
    bf16x8 fa[2][FM], fb[2][FN];
    int loa[TA::template nlo<FM>()], lob[TB::template nlo<FN>()];
#pragma unroll
    for (int x = 0; x < TA::template nlo<FM>(); ++x) loa[x] = TA::lane_offset(x, wm * TM, lane);
#pragma unroll
    for (int x = 0; x < TB::template nlo<FN>(); ++x) lob[x] = TB::lane_offset(x, wn * TN, lane);
    auto read_frags = [&](const char* sa, const char* sb, int ks, int slot) {
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[slot][j] = TB::frag(sb, lob, j, ks);
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[slot][i] = TA::frag(sa, loa, i, ks);
    };
    auto mfmas = [&](int slot) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
    };
    constexpr int WAIT_STRICT = (WAIT_KEEP & 15) | ((WAIT_KEEP >> 4) << 14) | 0x0070;   // vmcnt(WAIT_KEEP) lgkmcnt(0)
    // Stores of a tile's epilogue sit in the in-order memory queue in front of the next tile's fourth
    // stage.  The first two steps of a tile need stages 1 and 2 only, which the epilogue has already
    // waited for (see store_tile), so they run on a barrier alone (NOWAIT) and the stores drain
    // underneath them; the third step is the first to wait on the queue again, and its "all but the
    // two youngest stages" then covers the stores as well.
    constexpr int WAIT_LDS_ONLY = 0xC07F;   // lgkmcnt(0), vmcnt untouched
    auto step = [&](auto cur, auto nowait) {
        constexpr int CUR = decltype(cur)::value;
        constexpr bool NOWAIT = decltype(nowait)::value;
        using Nxt = std::integral_constant<int, (CUR + 1) % NST>;
        using Dst = std::integral_constant<int, (CUR + NST - 1) % NST>;
        issue(stA(Dst{}), stB(Dst{}));
        read_frags(stA(cur), stB(cur), 1, 1);
        mfmas(0);
        pace<FM * FN, NDS, NVM>();
        __builtin_amdgcn_s_waitcnt(NOWAIT ? WAIT_LDS_ONLY : WAIT_STRICT);
        __builtin_amdgcn_s_barrier();
        read_frags(stA(Nxt{}), stB(Nxt{}), 0, 0);
        mfmas(1);
        pace<FM * FN, NDS, 0>();
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    using Wait = std::false_type;
    using NoWait = std::true_type;
    static_assert(NST == 4, "the tile loop below is written for four stages");

    static_for<NST - 1>([&](auto i) { issue(stA(i), stB(i)); });
    __builtin_amdgcn_s_waitcnt(0x0070);   // all three stages landed: the first tile starts like every other
    __builtin_amdgcn_s_barrier();
    read_frags(sA0, sB0, 0, 0);

    for (int cv = first; cv < nblk;) {
        const TileCoord tc = map_tile(cv, nblk, tm, tn, p.groups, order);
        const GemmShard s = p.s[tc.g];
        const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
        const int rounds = s.kk / (BKT * NST);
        const int nv = next_valid(cv + G);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
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
        step(I0{}, NoWait{});
        if (rounds == 1) switch_tile();
        step(I1{}, NoWait{});
        step(I2{}, Wait{});
        step(I3{}, Wait{});
        for (int r = 1; r < rounds; ++r) {
            step(I0{}, Wait{});
            if (r == rounds - 1) switch_tile();
            step(I1{}, Wait{});
            step(I2{}, Wait{});
            step(I3{}, Wait{});
        }
        store_tile<BM, BN, TM, TN, FM, FN, EPI, OutT, true>(acc, s, m0, n0, wm, wn, lane, sOut);
        cv = nv;
    }
    __builtin_amdgcn_s_waitcnt(0x0070);   // trailing (unused) loads must land before LDS is released
}

// ------------------------------------------------------------------------------------------------
// The persistent kernel on v_mfma_f32_16x16x32_bf16.  Same tiles, stages, load stream, counters and
// barriers as gemm_mfma_persist_kernel; the matrix instruction spans the whole 32-deep stage, its
// accumulator block is 16 x 16 (four registers), and a step is split by row blocks instead of by
// reduction halves.  Under a sustained load of random operands the part's power management lets this
// instruction run at a higher clock than the 32x32x16 form (MFMA-only loop: 2070 against 1843 TFLOP/s).
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int NST, int EPI, typename OutT>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_persist16_kernel(GemmPlan p, int tm, int tn, int order, int nblk) {
    constexpr int BKT = 32;
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 16, FN = TN / 16;       // 16 x 16 blocks per wave
    static_assert(FM % 2 == 0, "the row blocks are multiplied in two halves");
    constexpr int HM = FM / 2;
    constexpr int NDS_A = A_KC ? HM : 2 * HM;                           // LDS reads of half the A fragments
    constexpr int NDS_B = B_KC ? FN : 2 * FN;                           // ... of all B fragments
    using TA = Tile<BM, A_KC, NT, BKT, true>;
    using TB = Tile<BN, B_KC, NT, BKT, true>;
    constexpr int NVM = TA::PER_THREAD + TB::PER_THREAD;
    constexpr int WAIT_KEEP = (NST - 2) * NVM;
    static_assert(NST == 4, "written for four stages");
    __shared__ __attribute__((aligned(1024))) char sA0[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA1[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA2[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sA3[TA::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB0[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB1[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB2[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sB3[TB::BYTES];
    __shared__ __attribute__((aligned(1024))) char sOut[WM * WN * STAGE_BYTES];   // epilogue windows, one per wave
    auto stA = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sA0; else if constexpr (I == 1) return sA1; else if constexpr (I == 2) return sA2; else return sA3;
    };
    auto stB = [&](auto i) -> char* {
        constexpr int I = decltype(i)::value;
        if constexpr (I == 0) return sB0; else if constexpr (I == 1) return sB1; else if constexpr (I == 2) return sB2; else return sB3;
    };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int G = gridDim.x;

    // first valid tile at or after virtual block v (uneven shards have fewer tiles than tm x tn)
    auto next_valid = [&](int v) {
        for (; v < nblk; v += G) {
            const TileCoord tc = map_tile(v, nblk, tm, tn, p.groups, order);
            if (tc.valid && tc.tile_m * BM < p.s[tc.g].m && tc.tile_n * BN < p.s[tc.g].n) break;
        }
        return v;
    };

    // ---- load cursor: always exactly NST - 1 stages ahead of the compute cursor ------------------
    gbl_char* A = nullptr;
    gbl_char* B = nullptr;
    uint32_t offa[TA::PER_THREAD], offb[TB::PER_THREAD];
    uint32_t stepa = 0, stepb = 0;
    const int first = next_valid(blockIdx.x);
    if (first >= nblk) return;         // nothing for this workgroup
    auto open_tile = [&](int v) {
        const TileCoord tc = map_tile(v, nblk, tm, tn, p.groups, order);
        const GemmShard& s = p.s[tc.g];
        A = (gbl_char*)s.a;
        B = (gbl_char*)s.b;
        // the chunk positions are recomputed from the thread id at every tile: kept across the reduction loop
        // they would take registers that the loop does not have
        int t = tid;
        asm volatile("" : "+v"(t));
#pragma unroll
        for (int it = 0; it < TA::PER_THREAD; ++it) offa[it] = TA::src_offset(s.lda, tc.tile_m * BM, s.m, it * NT + t);
#pragma unroll
        for (int it = 0; it < TB::PER_THREAD; ++it) offb[it] = TB::src_offset(s.ldb, tc.tile_n * BN, s.n, it * NT + t);
        stepa = TA::step_bytes(s.lda);
        stepb = TB::step_bytes(s.ldb);
    };
    open_tile(first);
    // Branch-free: always NVM loads (the wait counts rely on it), then one stage forward.  Because a
    // tile has a multiple of NST stages, the cursor leaves a tile exactly after step 0 of the tile's
    // last round; the tile loop below re-opens it there.  Past the last tile the steps are zeroed, so
    // the last stage is simply re-read (in bounds, never used).
    auto issue = [&](char* da, char* db) {
        TA::load_direct_untracked(da, A, offa, wave);
        TB::load_direct_untracked(db, B, offb, wave);
        A += stepa;
        B += stepb;
    };

    // ---- compute side --------------------------------------------------------------------------
    // One v_mfma_f32_16x16x32_bf16 spans a whole 32-deep stage.  A step multiplies the upper half of the
    // row blocks, then the lower half: fa[0] / fa[1] hold the A fragments of the two halves, fb[slot] the
    // B fragments of a stage (slot = stage parity; both halves use them, so the next stage's go to the
    // other slot).
    f32x4 acc[FM][FN];
    bf16x8 fa[2][HM], fb[2][FN];
    static_assert((A_KC || (TM % 128 == 0 && FM <= 8)) && (B_KC || (TN % 64 == 0 && FN <= 4)), "see Tile::lane_offset16");
    const int loa = TA::lane_offset16(wm * TM, lane), lob = TB::lane_offset16(wn * TN, lane);
    auto read_a = [&](const char* sa, int half) {
#pragma unroll
        for (int i = 0; i < HM; ++i) fa[half][i] = TA::frag16(sa, loa, half * HM + i);
    };
    auto read_b = [&](const char* sb, int slot) {
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[slot][j] = TB::frag16(sb, lob, j);
    };
    auto mfmas = [&](int half, int slot) {
#pragma unroll
        for (int i = 0; i < HM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[half * HM + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[half][i], fb[slot][j], acc[half * HM + i][j], 0, 0, 0);
    };
    constexpr int WAIT_STRICT = (WAIT_KEEP & 15) | ((WAIT_KEEP >> 4) << 14) | 0x0070;   // vmcnt(WAIT_KEEP) lgkmcnt(0)
    // Stores of a tile's epilogue sit in the in-order memory queue in front of the next tile's fourth
    // stage.  The first two steps of a tile need stages 1 and 2 only, which the epilogue has already
    // waited for (see store_tile), so they run on a barrier alone (NOWAIT) and the stores drain
    // underneath them; the third step is the first to wait on the queue again, and its "all but the
    // two youngest stages" then covers the stores as well.
    constexpr int WAIT_LDS_ONLY = 0xC07F;   // lgkmcnt(0), vmcnt untouched
    auto step = [&](auto cur, auto nowait) {
        constexpr int CUR = decltype(cur)::value;
        constexpr bool NOWAIT = decltype(nowait)::value;
        using Nxt = std::integral_constant<int, (CUR + 1) % NST>;
        using Dst = std::integral_constant<int, (CUR + NST - 1) % NST>;
        issue(stA(Dst{}), stB(Dst{}));
        read_a(stA(cur), 1);
        mfmas(0, CUR & 1);
        pace<HM * FN, NDS_A, NVM>();
        __builtin_amdgcn_s_waitcnt(NOWAIT ? WAIT_LDS_ONLY : WAIT_STRICT);
        __builtin_amdgcn_s_barrier();
        read_a(stA(Nxt{}), 0);
        read_b(stB(Nxt{}), (CUR + 1) & 1);
        mfmas(1, CUR & 1);
        pace<HM * FN, NDS_A + NDS_B, 0>();
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    using Wait = std::false_type;
    using NoWait = std::true_type;
    static_assert(NST == 4, "the tile loop below is written for four stages");

    static_for<NST - 1>([&](auto i) { issue(stA(i), stB(i)); });
    __builtin_amdgcn_s_waitcnt(0x0070);   // all three stages landed: the first tile starts like every other
    __builtin_amdgcn_s_barrier();
    read_a(sA0, 0);
    read_b(sB0, 0);

    for (int cv = first; cv < nblk;) {
        const TileCoord tc = map_tile(cv, nblk, tm, tn, p.groups, order);
        const GemmShard s = p.s[tc.g];
        const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
        const int rounds = s.kk / (BKT * NST);
        const int nv = next_valid(cv + G);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;
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
        step(I0{}, NoWait{});
        if (rounds == 1) switch_tile();
        step(I1{}, NoWait{});
        step(I2{}, Wait{});
        step(I3{}, Wait{});
        for (int r = 1; r < rounds; ++r) {
            step(I0{}, Wait{});
            if (r == rounds - 1) switch_tile();
            step(I1{}, Wait{});
            step(I2{}, Wait{});
            step(I3{}, Wait{});
        }
        store_tile16<BM, BN, TM, TN, EPI, OutT>(acc, s, m0, n0, wm, wn, lane, sOut);
        cv = nv;
    }
    __builtin_amdgcn_s_waitcnt(0x0070);   // trailing (unused) loads must land before LDS is released
}

// ------------------------------------------------------------------------------------------------
// Rows 4 and 5 of Table 1 next to bf16 tensors: one operand is an un-reduced P(sum) partial (fp32),
// the other a bf16 B tensor, the result again fp32 partials.  Rounding the partial to bf16 would change
// the sum it stands for, so it is split exactly into three bf16 terms on its way into LDS,
//     x = hi + mid + lo,   hi = x cut to its top 16 bits, mid = (x - hi) cut likewise, lo = x - hi - mid
// (each remainder is exact in fp32 and lo fits 8 significant bits), and every reduction step runs three
// bf16 MFMAs, one per term, into the same fp32 accumulator.  Products of bf16 values are exact in
// fp32, so the result differs from an fp32 GEMM by accumulation order only.  (Inf in the partial gives
// NaN: inf - inf in the split.)
// 128 x 128 tile, 4 waves of 64 x 64 (16 blocks of v_mfma_f32_16x16x32_bf16), two LDS stages of 32 reduction elements: three term tiles of the
// fp32 operand (written from registers, same chunk order and swizzle as the direct-to-LDS image) and
// one tile of the bf16 operand (direct to LDS).  F32_B: the fp32 operand is B (row 5), else A (row 4).
// ------------------------------------------------------------------------------------------------
struct SplitTerms { u32x4 hi, mid, lo; };
__device__ inline SplitTerms split_f32x8(const f32x4 a, const f32x4 b) {
    uint32_t h[8], m[8], l[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x = e < 4 ? a[e] : b[e - 4];
        h[e] = __float_as_uint(x) & 0xFFFF0000u;
        const float r1 = x - __uint_as_float(h[e]);
        m[e] = __float_as_uint(r1) & 0xFFFF0000u;
        const float r2 = r1 - __uint_as_float(m[e]);
        l[e] = __float_as_uint(r2);   // at most 8 significant bits: the low half is zero
    }
    SplitTerms t;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        t.hi[d] = (h[2 * d] >> 16) | h[2 * d + 1];
        t.mid[d] = (m[2 * d] >> 16) | m[2 * d + 1];
        t.lo[d] = (l[2 * d] >> 16) | (l[2 * d + 1] & 0xFFFF0000u);
    }
    return t;
}

// HW: extent of the bf16 operand's side of the tile, 128 (4 waves) or 256 (8 waves).  The split costs about as many
// vector instructions per element of the fp32 operand as fit beside the matrix instructions of a 128-wide tile;
// with 256 every split element feeds twice as many of them and the bf16 operand is fetched half as often.
template <bool A_KC, bool B_KC, bool F32_B, int HW>
__global__ __launch_bounds__(HW * 2, HW == 256 ? 4 : 2) void gemm_split_kernel(GemmPlan p, int tm, int tn, int order) {
    constexpr int BM = F32_B ? HW : 128, BN = F32_B ? 128 : HW, WN = BN / 64, NT = HW * 2, BKT = 32;
    constexpr int TM = 64, TN = 64, FM = 4, FN = 4;   // 16 x 16 blocks of v_mfma_f32_16x16x32_bf16 (one per 32-deep stage)
    using TA = Tile<BM, A_KC, NT, BKT, true>;
    using TB = Tile<BN, B_KC, NT, BKT, true>;
    using TF = std::conditional_t<F32_B, TB, TA>;   // tile type of the fp32 operand
    using TH = std::conditional_t<F32_B, TA, TB>;   // ... of the bf16 operand
    // two stages of three term tiles (hi, mid, lo); after the reduction loop the same memory serves as the
    // epilogue's per-wave windows, so that two workgroups fit a compute unit's LDS with either tile
    __shared__ __attribute__((aligned(1024))) char sFF[2][3][TF::BYTES];
    __shared__ __attribute__((aligned(1024))) char sH0[TH::BYTES];
    __shared__ __attribute__((aligned(1024))) char sH1[TH::BYTES];
    static_assert(sizeof(sFF) >= (NT / 64) * STAGE_BYTES, "epilogue windows fit the term tiles");
    char (*sF0)[TF::BYTES] = sFF[0];
    char (*sF1)[TF::BYTES] = sFF[1];
    char* sOut = &sFF[0][0][0];

    const TileCoord tc = map_tile(blockIdx.x, gridDim.x, tm, tn, p.groups, order);
    if (!tc.valid) return;
    const GemmShard s = p.s[tc.g];
    const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
    if (m0 >= s.m || n0 >= s.n) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // fp32 operand: 32 bytes per chunk (twice the bf16 byte offset); bf16 operand: direct to LDS
    const char* F = static_cast<const char*>(F32_B ? s.b : s.a);
    gbl_char* H = (gbl_char*)(F32_B ? s.a : s.b);
    const int ldf = F32_B ? s.ldb : s.lda, ldh = F32_B ? s.lda : s.ldb;
    uint64_t offf[TF::PER_THREAD];
    uint32_t offh[TH::PER_THREAD];
#pragma unroll
    for (int it = 0; it < TF::PER_THREAD; ++it)
        offf[it] = (uint64_t)2 * TF::src_offset(ldf, F32_B ? n0 : m0, F32_B ? s.n : s.m, it * NT + tid);
#pragma unroll
    for (int it = 0; it < TH::PER_THREAD; ++it) offh[it] = TH::src_offset(ldh, F32_B ? m0 : n0, F32_B ? s.m : s.n, it * NT + tid);
    const uint64_t stepf = (uint64_t)2 * TF::step_bytes(ldf);
    const uint32_t steph = TH::step_bytes(ldh);

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;
    const int loa = TA::lane_offset16(wm * TM, lane), lob = TB::lane_offset16(wn * TN, lane);

    f32x4 raw[TF::PER_THREAD][2];
    auto fetch = [&]() {   // global -> registers (fp32 operand), global -> LDS (bf16 operand)
#pragma unroll
        for (int it = 0; it < TF::PER_THREAD; ++it) {
            const f32x4* g = reinterpret_cast<const f32x4*>(F + offf[it]);
            raw[it][0] = g[0];
            raw[it][1] = g[1];
        }
    };
    auto stash = [&](char (*dst)[TF::BYTES]) {   // registers -> three term tiles
#pragma unroll
        for (int it = 0; it < TF::PER_THREAD; ++it) {
            const SplitTerms t = split_f32x8(raw[it][0], raw[it][1]);
            const int pos = (it * NT + tid) * 16;
            *reinterpret_cast<u32x4*>(dst[0] + pos) = t.hi;
            *reinterpret_cast<u32x4*>(dst[1] + pos) = t.mid;
            *reinterpret_cast<u32x4*>(dst[2] + pos) = t.lo;
        }
    };
    auto compute = [&](const char (*sf)[TF::BYTES], const char* sh) {
        if constexpr (F32_B) {
            bf16x8 fa[FM];
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[i] = TA::frag16(sh, loa, i);
#pragma unroll
            for (int term = 0; term < 3; ++term)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const bf16x8 fb = TB::frag16(sf[term], lob, j);
#pragma unroll
                    for (int i = 0; i < FM; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb, acc[i][j], 0, 0, 0);
                }
        } else {
            bf16x8 fb[FN];
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = TB::frag16(sh, lob, j);
#pragma unroll
            for (int term = 0; term < 3; ++term)
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    const bf16x8 fa = TA::frag16(sf[term], loa, i);
#pragma unroll
                    for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb[j], acc[i][j], 0, 0, 0);
                }
        }
    };

    const int steps = s.kk / BKT;
    fetch();
    TH::load_direct(sH0, H, offh, wave);
    stash(sF0);
    __builtin_amdgcn_s_waitcnt(0x0070);
    __syncthreads();
    // stage names are compile-time in every step, so that the compiler can tell the direct-to-LDS
    // load into one stage from the fragment reads of the other
    auto step = [&](auto cur, bool more) {   // `more` is uniform
        constexpr int CUR = decltype(cur)::value;
        if (more) {
            F += stepf;
            H += steph;
            fetch();
            TH::load_direct(CUR ? sH0 : sH1, H, offh, wave);
        }
        compute(CUR ? sF1 : sF0, CUR ? sH1 : sH0);
        if (more) {
            stash(CUR ? sF0 : sF1);
            // Scheduling hint: the vector instructions that split the next stage's fp32 values go a few behind each of
            // this stage's matrix instructions instead of in a block after them (the matrix pipe runs an instruction
            // for 16 cycles while the wave may issue others).  Which matrix instructions take them is by measurement
            // (ms on [4096,4096] x [4096,1024] per device, 8 devices; no hint / behind all 48 / behind the last 32,
            // i.e. not the first term's): fp32 A, wide tile .673 / .645 / .606, narrow .784 / .791 / .735;
            // fp32 B, wide .736 / .687 / .749, narrow .862 / .866 / .833.
            constexpr int FIRST = (F32_B && HW == 256) ? 0 : FM * FN;
            constexpr int PER = ((F32_B && HW == 256) ? 2 : 3) * TF::PER_THREAD;
            static_for<3 * FM * FN>([&](auto i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                             // 1 MFMA
                if constexpr (decltype(i)::value >= FIRST) __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);   // vector ALU
            });
        }
        __builtin_amdgcn_s_waitcnt(0x0070);   // this wave's direct-to-LDS loads have landed
        __syncthreads();                      // next stage complete, this one free
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    for (int t = 0; t + 1 < steps; t += 2) {
        step(I0{}, true);
        step(I1{}, t + 2 < steps);
    }
    if (steps & 1) step(I0{}, false);
    // every step ends with a workgroup barrier: nobody reads the term tiles any more
    store_tile16<BM, BN, TM, TN, SBP_EPI_NONE, float>(acc, s, m0, n0, wm, wn, lane, sOut);
}

template <bool F32_B, int HW>
int32_t launch_split_cfg(const GemmPlan& plan, int max_m, int max_n, hipStream_t st) {
    constexpr int BM = F32_B ? HW : 128, BN = F32_B ? 128 : HW;
    const int tm = (max_m + BM - 1) / BM, tn = (max_n + BN - 1) / BN;
    const int64_t nblk = ((int64_t)tm * tn * plan.groups + 7) / 8 * 8;
    if (nblk > 0x7FFFFFFF) return SBP_ERR_UNSUPPORTED;
    void (*kern)(GemmPlan, int, int, int);
    if (plan.a_kc && plan.b_kc) kern = gemm_split_kernel<true, true, F32_B, HW>;
    else if (plan.a_kc) kern = gemm_split_kernel<true, false, F32_B, HW>;
    else if (plan.b_kc) kern = gemm_split_kernel<false, true, F32_B, HW>;
    else kern = gemm_split_kernel<false, false, F32_B, HW>;
    hipLaunchKernelGGL(kern, dim3((uint32_t)nblk), dim3(HW * 2), 0, st, plan, tm, tn, tile_order_for(tm, tn));
    return launch_status(__func__);
}

// The wide tile when the bf16 operand's side has at least 256 rows or columns and the narrow tiling would
// still leave every compute unit several workgroups; `variant` 31 / 32 force the narrow / the wide tile.
template <bool F32_B>
int32_t launch_split(const GemmPlan& plan, int max_m, int max_n, int variant, hipStream_t st) {
    const int hside = F32_B ? max_m : max_n;
    const int64_t wide_tiles = (int64_t)((max_m + (F32_B ? 255 : 127)) / (F32_B ? 256 : 128)) * ((max_n + (F32_B ? 127 : 255)) / (F32_B ? 128 : 256)) * plan.groups;
    const bool wide = variant == 32 || (variant != 31 && hside >= 256 && wide_tiles >= 2 * (int64_t)compute_units());
    return wide ? launch_split_cfg<F32_B, 256>(plan, max_m, max_n, st) : launch_split_cfg<F32_B, 128>(plan, max_m, max_n, st);
}

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int ODD, int EPI, typename OutT>
int32_t launch_mfma_cfg(const GemmPlan& plan, int max_m, int max_n, hipStream_t st) {
    const int tm = (max_m + BM - 1) / BM, tn = (max_n + BN - 1) / BN;
    const int64_t tiles = (int64_t)tm * tn * plan.groups;
    const int64_t nblk = (tiles + 7) / 8 * 8;
    if (nblk > 0x7FFFFFFF) return SBP_ERR_UNSUPPORTED;
    if constexpr (ODD >= 100) {   // persistent kernel, ODD - 100 stages
        int grid = compute_units() / 8 * 8;
        if (grid > nblk) grid = (int)nblk;
        if constexpr (ODD >= 200)
            hipLaunchKernelGGL((gemm_mfma_persist16_kernel<BM, BN, WM, WN, A_KC, B_KC, ODD - 200, EPI, OutT>), dim3((uint32_t)grid),
                               dim3(WM * WN * 64), 0, st, plan, tm, tn, tile_order_for(tm, tn) & 0xFFFF, (int)nblk);
        else
            hipLaunchKernelGGL((gemm_mfma_persist_kernel<BM, BN, WM, WN, A_KC, B_KC, ODD - 100, EPI, OutT>), dim3((uint32_t)grid),
                               dim3(WM * WN * 64), 0, st, plan, tm, tn, tile_order_for(tm, tn) & 0xFFFF, (int)nblk);
        return launch_status(__func__);
    }
    void (*kern)(GemmPlan, int, int, int);
    if constexpr (ODD >= 100) kern = nullptr;
    else if constexpr (ODD >= 50) kern = gemm_mfma_pipe16_kernel<BM, BN, WM, WN, A_KC, B_KC, ODD - 50, EPI, OutT>;   // 16x16x32 instruction
    else if constexpr (ODD >= 3) kern = gemm_mfma_pipe_kernel<BM, BN, WM, WN, A_KC, B_KC, ODD, EPI, OutT>;   // ODD carries the stage count
    else kern = gemm_mfma_kernel<BM, BN, WM, WN, A_KC, B_KC, 0, EPI, OutT>;
    hipLaunchKernelGGL(kern, dim3((uint32_t)nblk), dim3(WM * WN * 64), 0, st, plan, tm, tn, tile_order_for(tm, tn));
    return launch_status(__func__);
}

template <int BM, int BN, int WM, int WN, int ODD, int EPI, typename OutT>
int32_t launch_mfma_layout(const GemmPlan& plan, int max_m, int max_n, hipStream_t st) {
    if (plan.a_kc && plan.b_kc) return launch_mfma_cfg<BM, BN, WM, WN, true, true, ODD, EPI, OutT>(plan, max_m, max_n, st);
    if (plan.a_kc) return launch_mfma_cfg<BM, BN, WM, WN, true, false, ODD, EPI, OutT>(plan, max_m, max_n, st);
    if (plan.b_kc) return launch_mfma_cfg<BM, BN, WM, WN, false, true, ODD, EPI, OutT>(plan, max_m, max_n, st);
    return launch_mfma_cfg<BM, BN, WM, WN, false, false, ODD, EPI, OutT>(plan, max_m, max_n, st);
}

// fp32 results carry no epilogue on this path (GeLU of a P(sum) partial is rejected upstream and
// fp32 inputs take the generic kernel), so three (epilogue, output) pairs cover every request.
template <int BM, int BN, int WM, int WN, int ODD>
int32_t launch_mfma_out(const GemmPlan& plan, int max_m, int max_n, hipStream_t st) {
    if (plan.out_dtype == SBP_F32) {
        if (plan.epilogue != SBP_EPI_NONE) return SBP_ERR_UNSUPPORTED;
        return launch_mfma_layout<BM, BN, WM, WN, ODD, SBP_EPI_NONE, float>(plan, max_m, max_n, st);
    }
    if (plan.epilogue == SBP_EPI_GELU) return launch_mfma_layout<BM, BN, WM, WN, ODD, SBP_EPI_GELU, uint16_t>(plan, max_m, max_n, st);
    return launch_mfma_layout<BM, BN, WM, WN, ODD, SBP_EPI_NONE, uint16_t>(plan, max_m, max_n, st);
}

template <bool A_BF16, bool B_BF16, typename OutT>
void launch_generic_epi(const GemmPlan& plan, dim3 grid, hipStream_t st) {
    if (plan.epilogue == SBP_EPI_GELU)
        hipLaunchKernelGGL((gemm_generic_kernel<A_BF16, B_BF16, OutT, SBP_EPI_GELU>), grid, dim3(16, 16), 0, st, plan);
    else
        hipLaunchKernelGGL((gemm_generic_kernel<A_BF16, B_BF16, OutT, SBP_EPI_NONE>), grid, dim3(16, 16), 0, st, plan);
}

// Shapes the MFMA kernel takes: whole 64-element reduction steps, 16-byte aligned rows.
bool mfma_ok(const GemmPlan& plan) {
    if (plan.in_dtype != SBP_BF16) return false;
    for (int g = 0; g < plan.groups; ++g) {
        const GemmShard& s = plan.s[g];
        if (s.m == 0 || s.n == 0) continue;
        if (s.kk == 0 || s.kk % BK) return false;
        if (s.lda % 8 || s.ldb % 8) return false;
        if (!plan.a_kc && s.m < 8) return false;
        if (!plan.b_kc && s.n < 8) return false;
        // source offsets are 32-bit byte offsets from the shard base
        const int64_t ea = plan.a_kc ? (int64_t)s.m * s.lda : (int64_t)s.kk * s.lda;
        const int64_t eb = plan.b_kc ? (int64_t)s.n * s.ldb : (int64_t)s.kk * s.ldb;
        if (ea * 2 >= ((int64_t)1 << 32) || eb * 2 >= ((int64_t)1 << 32)) return false;
    }
    return true;
}

// Shapes the split kernel takes: whole 32-element reduction steps, 16-byte aligned rows of both operands.
bool split_ok(const GemmPlan& plan) {
    if (plan.in_dtype != SBP_BF16 || plan.out_dtype != SBP_F32 || plan.epilogue != SBP_EPI_NONE) return false;
    const bool fb = plan.f32_operand == 2;
    for (int g = 0; g < plan.groups; ++g) {
        const GemmShard& s = plan.s[g];
        if (s.m == 0 || s.n == 0) continue;
        if (s.kk == 0 || s.kk % 32) return false;
        if ((fb ? s.lda : s.ldb) % 8 || (fb ? s.ldb : s.lda) % 4) return false;
        if (!plan.a_kc && (s.m < 8 || (!fb && s.m % 4))) return false;
        if (!plan.b_kc && (s.n < 8 || (fb && s.n % 4))) return false;
        const int64_t ea = plan.a_kc ? (int64_t)s.m * s.lda : (int64_t)s.kk * s.lda;
        const int64_t eb = plan.b_kc ? (int64_t)s.n * s.ldb : (int64_t)s.kk * s.ldb;
        if (ea * 2 >= ((int64_t)1 << 32) || eb * 2 >= ((int64_t)1 << 32)) return false;
    }
    return true;
}

// Which persistent kernel for a shape both take.  Measured (ms, lockstep / ping-pong): reduction length 512 with
// 61 tiles per compute unit 1.42 / 1.35; 2048 with 16 tiles 1.00 / 1.00, with 2 tiles 0.121 / 0.135; 4096 with 8
// tiles 0.93 / 0.93.  Short reductions gain (the tile change is cheaper), few tiles per unit lose.
bool pingpong_pays(const GemmPlan& plan, int max_m, int max_n) {
    int max_k = 0;
    for (int g = 0; g < plan.groups; ++g)
        if (plan.s[g].m && plan.s[g].n && plan.s[g].kk > max_k) max_k = plan.s[g].kk;
    const int64_t tiles = (int64_t)((max_m + 255) / 256) * ((max_n + 255) / 256) * plan.groups;
    return max_k <= 1024 && tiles >= 4 * (int64_t)compute_units();
}

}  // namespace

void set_tile_order(int32_t order) { g_tile_order.store(order, std::memory_order_relaxed); }

int compute_units() {
    constexpr int MAX_DEV = 64;
    static std::atomic<int> cached[MAX_DEV];   // 0 = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

int32_t launch_gemm(const GemmPlan& plan, int32_t variant, hipStream_t stream) {
    int max_m = 0, max_n = 0;
    for (int g = 0; g < plan.groups; ++g) {
        if (plan.s[g].m == 0 || plan.s[g].n == 0) continue;
        max_m = plan.s[g].m > max_m ? plan.s[g].m : max_m;
        max_n = plan.s[g].n > max_n ? plan.s[g].n : max_n;
    }
    // the fused row maximum exists in the persistent bf16 kernel only; the caller does anything else in two passes
    if (plan.epilogue == EPI_ROWMAX && (max_m == 0 || max_n == 0 || plan.f32_operand || variant == 1 || !mfma_ok(plan)))
        return SBP_ERR_UNSUPPORTED;
    if (max_m == 0 || max_n == 0) return SBP_OK;   // every local product is empty
    // variants 31 / 32 choose the tile of the split kernel only; every other product takes the default path
    if ((variant == 31 || variant == 32) && !(plan.f32_operand && split_ok(plan))) variant = 0;

    if (plan.f32_operand) {
        // Table 1 rows 4 / 5 with a bf16 partner: split kernel, else the generic kernel with mixed element types
        if (variant != 1 && split_ok(plan)) {
            if (variant > 1 && variant != 31 && variant != 32) return SBP_ERR_UNSUPPORTED;
            return plan.f32_operand == 2 ? launch_split<true>(plan, max_m, max_n, variant, stream) : launch_split<false>(plan, max_m, max_n, variant, stream);
        }
        if (variant > 1) return SBP_ERR_UNSUPPORTED;
        const dim3 grid((max_n + 15) / 16, (max_m + 15) / 16, plan.groups);
        if (grid.y > 65535 || grid.z > 65535) return SBP_ERR_UNSUPPORTED;
        if (plan.out_dtype != SBP_F32 || plan.epilogue != SBP_EPI_NONE) return SBP_ERR_DTYPE;
        if (plan.f32_operand == 2) launch_generic_epi<true, false, float>(plan, grid, stream);
        else launch_generic_epi<false, true, float>(plan, grid, stream);
        return launch_status(__func__);
    }
    const bool fast = mfma_ok(plan);
    if (variant == 1 || !fast) {
        if (variant > 1) return SBP_ERR_UNSUPPORTED;   // a forced MFMA variant cannot take this shape
        const dim3 grid((max_n + 15) / 16, (max_m + 15) / 16, plan.groups);
        if (grid.y > 65535 || grid.z > 65535) return SBP_ERR_UNSUPPORTED;
        if (plan.in_dtype == SBP_BF16) {
            if (plan.out_dtype == SBP_F32) launch_generic_epi<true, true, float>(plan, grid, stream);
            else launch_generic_epi<true, true, uint16_t>(plan, grid, stream);
        } else {
            if (plan.out_dtype != SBP_F32) return SBP_ERR_DTYPE;
            launch_generic_epi<false, false, float>(plan, grid, stream);
        }
        return launch_status(__func__);
    }
    bool k128 = true;   // every local reduction a whole number of four-stage rounds
    for (int g = 0; g < plan.groups; ++g)
        if (plan.s[g].m && plan.s[g].n && plan.s[g].kk % 128) k128 = false;
    if (plan.epilogue == EPI_ROWMAX) {
        // fused row maximum: persistent bf16 kernel only; anything else is done in two passes by the caller
        if (!(k128 && max_m > 128 && max_n > 128 && plan.out_dtype == SBP_BF16 && (variant == 0 || variant == 12 || variant == 16 || variant == 21))) return SBP_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(fill_rowmax_kernel, dim3((uint32_t)((max_m + 255) / 256), (uint32_t)plan.groups), dim3(256), 0, stream, plan);
        const int32_t st = launch_status(__func__);
        if (st != SBP_OK) return st;
        if (variant == 12) return launch_mfma_layout<256, 256, 2, 4, 104, EPI_ROWMAX, uint16_t>(plan, max_m, max_n, stream);
        if (variant == 21 || (variant == 0 && pingpong_pays(plan, max_m, max_n))) {
            const int tm = (max_m + 255) / 256, tn = (max_n + 255) / 256;
            return launch_gemm_pingpong(plan, max_m, max_n, tile_order_for(tm, tn) & 0xFFFF, stream);
        }
        return launch_mfma_layout<256, 256, 2, 4, 204, EPI_ROWMAX, uint16_t>(plan, max_m, max_n, stream);
    }
    if (variant == 0) {
        // Default: the 256 x 256 tile over 8 waves with four 32-deep LDS stages, as one persistent
        // workgroup per compute unit when the reduction length allows it; shapes that would leave most
        // of such a tile empty take the 128 x 128 tile.  The persistent kernel runs on the 16x16x32
        // matrix instruction.
        variant = (max_m > 128 && max_n > 128) ? (k128 ? (pingpong_pays(plan, max_m, max_n) ? 21 : 16) : 7) : 4;
    }
    switch (variant) {
        case 3: return launch_mfma_out<256, 256, 2, 4, 0>(plan, max_m, max_n, stream);
        case 4: return launch_mfma_out<128, 128, 2, 2, 0>(plan, max_m, max_n, stream);
        case 6: return launch_mfma_out<256, 256, 2, 4, 4>(plan, max_m, max_n, stream);
        case 7: return launch_mfma_out<256, 256, 2, 4, 54>(plan, max_m, max_n, stream);
        case 12: return k128 ? launch_mfma_out<256, 256, 2, 4, 104>(plan, max_m, max_n, stream) : SBP_ERR_UNSUPPORTED;
        case 16: return k128 ? launch_mfma_out<256, 256, 2, 4, 204>(plan, max_m, max_n, stream) : SBP_ERR_UNSUPPORTED;
        case 21: {
            if (!k128) return SBP_ERR_UNSUPPORTED;
            const int tm = (max_m + 255) / 256, tn = (max_n + 255) / 256;
            return launch_gemm_pingpong(plan, max_m, max_n, tile_order_for(tm, tn) & 0xFFFF, stream);
        }
        default: return SBP_ERR_UNSUPPORTED;
    }
}

}  // namespace sbp
