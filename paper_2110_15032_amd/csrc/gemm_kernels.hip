// Grouped per-shard GEMM for sbp_matmul (paper Sec. 3.1, Table 1): device g computes
// C_g = A_g B_g from the local tensors it holds; all k devices run in ONE launch.
//
//   gemm_generic_kernel   any dtype / shape / pitch, one output element per lane, fp32 FMA chain.
//                         Used for fp32 operands and for shapes the MFMA path does not take.
//   gemm_mfma_kernel      bf16 x bf16 -> fp32 on the matrix cores (v_mfma_f32_32x32x16_bf16),
//                         BM x BN x 64 macro-tile per workgroup, double-buffered LDS.
//
// Operand storage: "KC" = reduction index contiguous ([m][kk] for A, [n][kk] for B), otherwise the
// reduction index is the slow one ([kk][m], [kk][n]).  Row-major X and W give A KC and B not-KC.
#include "sbp_internal.h"

namespace sbp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even, NaN kept quiet
__device__ inline uint16_t f32_to_bf16(float f) {
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// 0.5 x (1 + erf(x / sqrt 2)) written with erfc so that the negative tail keeps its relative accuracy
__device__ inline float gelu_erf(float x) { return 0.5f * x * erfcf(x * -0.70710678118654752f); }

template <int EPI>
__device__ inline float epilogue(float v) {
    if constexpr (EPI == SBP_EPI_GELU) return gelu_erf(v);
    else return v;
}

__device__ inline void store_out(float* c, int64_t pos, float v) { c[pos] = v; }
__device__ inline void store_out(uint16_t* c, int64_t pos, float v) { c[pos] = f32_to_bf16(v); }

// ------------------------------------------------------------------------------------------------
// generic kernel
// ------------------------------------------------------------------------------------------------
template <bool IN_BF16, typename OutT, int EPI>
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
        if constexpr (IN_BF16) {
            a = bf16_to_f32(static_cast<const uint16_t*>(s.a)[ia]);
            b = bf16_to_f32(static_cast<const uint16_t*>(s.b)[ib]);
        } else {
            a = static_cast<const float*>(s.a)[ia];
            b = static_cast<const float*>(s.b)[ib];
        }
        acc = fmaf(a, b, acc);
    }
    store_out(static_cast<OutT*>(s.c), (int64_t)m * s.ldc + n, epilogue<EPI>(acc));
}

// ------------------------------------------------------------------------------------------------
// MFMA kernel
// ------------------------------------------------------------------------------------------------
constexpr int BK = 64;  // reduction extent of one LDS stage, in elements (128 B per KC row)

// XOR swizzle of the eight 16-byte chunks of a 128-byte KC row.  Any 8 consecutive rows land in 8
// different chunk slots, and rows r, r + 8 differ as well, so a column of fragments read with
// ds_read_b128 spreads over all banks whether the LDS serves 128 or 256 bytes per clock.
__device__ inline int swz(int row) { return (row ^ (row >> 3)) & 7; }

template <int R, bool KC, int NT>
struct Tile {
    static constexpr int BYTES = R * BK * 2;
    static constexpr int CHUNKS = BYTES / 16;
    static constexpr int PER_THREAD = CHUNKS / NT;
    static_assert(CHUNKS % NT == 0, "tile must divide over the workgroup");

    // global -> registers.  first = first tile row (m or n index), limit = extent of that index.
    __device__ static void fetch(u32x4 (&reg)[PER_THREAD], const uint16_t* base, int ld, int first, int limit,
                                 int k0, int tid) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int q = tid + it * NT;
            const uint16_t* ptr;
            if constexpr (KC) {
                int row = first + (q >> 3);
                row = row < limit ? row : limit - 1;                 // clamped rows are never stored
                ptr = base + (int64_t)row * ld + k0 + (q & 7) * 8;
            } else {
                constexpr int CPR = R / 8;                           // chunks per kk-row
                int col = first + (q % CPR) * 8;
                col = col < limit ? col : limit - 8;
                ptr = base + (int64_t)(k0 + q / CPR) * ld + col;
            }
            reg[it] = *reinterpret_cast<const u32x4*>(ptr);
        }
    }
    // registers -> LDS
    __device__ static void stash(const u32x4 (&reg)[PER_THREAD], char* lds, int tid) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int q = tid + it * NT;
            int off;
            if constexpr (KC) {
                const int row = q >> 3;
                off = row * 128 + (((q & 7) ^ swz(row)) << 4);
            } else {
                off = q * 16;                                        // [kk][R] dense
            }
            *reinterpret_cast<u32x4*>(lds + off) = reg[it];
        }
    }
    // LDS -> one MFMA operand: 8 consecutive kk (16 s + 8 (lane / 32) ...) for index `row`
    __device__ static bf16x8 frag(const char* lds, int row, int s, int lane) {
        const int kh = lane >> 5;
        if constexpr (KC) {
            return *reinterpret_cast<const bf16x8*>(lds + row * 128 + (((2 * s + kh) ^ swz(row)) << 4));
        } else {
            const uint16_t* t = reinterpret_cast<const uint16_t*>(lds) + (16 * s + 8 * kh) * R + row;
            u16x8 v;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = t[j * R];
            return __builtin_bit_cast(bf16x8, v);
        }
    }
};

struct TileCoord {
    int g, tile_m, tile_n;
    bool valid;
};

// Workgroup id -> (shard, tile).  Hardware hands consecutive workgroup ids to the 8 XCDs in turn;
// re-linearise so that each XCD walks a contiguous range of tiles (with k = 8 one whole shard,
// whose W_g then lives in that XCD's L2 only), and walk the tiles of a shard in column-major
// groups of 8 tile-rows so that the 32 CUs of an XCD work on a compact patch at any time.
__device__ inline TileCoord map_tile(int bid, int nblk, int tm, int tn, int groups) {
    const int per_xcd = nblk >> 3;
    const int v = (bid & 7) * per_xcd + (bid >> 3);
    const int per_group = tm * tn;
    TileCoord t;
    t.valid = v < per_group * groups;
    t.g = v / per_group;
    const int tl = v - t.g * per_group;
    constexpr int GM = 8;
    const int band = tl / (GM * tn);
    const int first_m = band * GM;
    const int gsz = (tm - first_m) < GM ? (tm - first_m) : GM;
    const int in_band = tl - band * GM * tn;
    t.tile_m = first_m + in_band % gsz;
    t.tile_n = in_band / gsz;
    return t;
}

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int EPI, typename OutT>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(GemmPlan p, int tm, int tn) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;   // wave tile
    constexpr int FM = TM / 32, FN = TN / 32;   // 32x32 MFMA tiles per wave
    using TA = Tile<BM, A_KC, NT>;
    using TB = Tile<BN, B_KC, NT>;
    constexpr int STAGE = TA::BYTES + TB::BYTES;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const TileCoord tc = map_tile(blockIdx.x, gridDim.x, tm, tn, p.groups);
    if (!tc.valid) return;
    const GemmShard s = p.s[tc.g];
    const int m0 = tc.tile_m * BM, n0 = tc.tile_n * BN;
    if (m0 >= s.m || n0 >= s.n) return;   // uneven shards: this one has fewer tiles

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const uint16_t* A = static_cast<const uint16_t*>(s.a);
    const uint16_t* B = static_cast<const uint16_t*>(s.b);

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4 ra[TA::PER_THREAD], rb[TB::PER_THREAD];
    const int steps = s.kk / BK;
    TA::fetch(ra, A, s.lda, m0, s.m, 0, tid);
    TB::fetch(rb, B, s.ldb, n0, s.n, 0, tid);
    TA::stash(ra, smem, tid);
    TB::stash(rb, smem + TA::BYTES, tid);
    __syncthreads();

    for (int t = 0; t < steps; ++t) {
        const char* sa = smem + (t & 1) * STAGE;
        const char* sb = sa + TA::BYTES;
        if (t + 1 < steps) {
            TA::fetch(ra, A, s.lda, m0, s.m, (t + 1) * BK, tid);
            TB::fetch(rb, B, s.ldb, n0, s.n, (t + 1) * BK, tid);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[i] = TA::frag(sa, wm * TM + i * 32 + (lane & 31), ks, lane);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = TB::frag(sb, wn * TN + j * 32 + (lane & 31), ks, lane);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (t + 1 < steps) {
            char* da = smem + ((t + 1) & 1) * STAGE;
            TA::stash(ra, da, tid);
            TB::stash(rb, da + TA::BYTES, tid);
        }
        __syncthreads();
    }

    // D[8 (r / 4) + 4 (lane / 32) + r % 4][lane % 32] = acc[r]
    OutT* C = static_cast<OutT*>(s.c);
    const int cn = lane & 31, rm = 4 * (lane >> 5);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int n = n0 + wn * TN + j * 32 + cn;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * TM + i * 32 + 8 * (r >> 2) + rm + (r & 3);
                if (m < s.m && n < s.n) store_out(C, (int64_t)m * s.ldc + n, epilogue<EPI>(acc[i][j][r]));
            }
        }
}

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int EPI, typename OutT>
int32_t launch_mfma_cfg(const GemmPlan& plan, int max_m, int max_n, hipStream_t st) {
    auto kern = gemm_mfma_kernel<BM, BN, WM, WN, A_KC, B_KC, EPI, OutT>;
    constexpr int smem = 2 * (BM + BN) * BK * 2;
    static bool attr_set = false;   // benign race: the call is idempotent
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return SBP_ERR_LAUNCH;
        attr_set = true;
    }
    const int tm = (max_m + BM - 1) / BM, tn = (max_n + BN - 1) / BN;
    const int64_t tiles = (int64_t)tm * tn * plan.groups;
    const int64_t nblk = (tiles + 7) / 8 * 8;
    if (nblk > 0x7FFFFFFF) return SBP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3((uint32_t)nblk), dim3(WM * WN * 64), smem, st, plan, tm, tn);
    return hipGetLastError() == hipSuccess ? SBP_OK : SBP_ERR_LAUNCH;
}

template <int BM, int BN, int WM, int WN, int EPI, typename OutT>
int32_t launch_mfma_layout(const GemmPlan& plan, int max_m, int max_n, hipStream_t st) {
    if (plan.a_kc && plan.b_kc) return launch_mfma_cfg<BM, BN, WM, WN, true, true, EPI, OutT>(plan, max_m, max_n, st);
    if (plan.a_kc) return launch_mfma_cfg<BM, BN, WM, WN, true, false, EPI, OutT>(plan, max_m, max_n, st);
    if (plan.b_kc) return launch_mfma_cfg<BM, BN, WM, WN, false, true, EPI, OutT>(plan, max_m, max_n, st);
    return launch_mfma_cfg<BM, BN, WM, WN, false, false, EPI, OutT>(plan, max_m, max_n, st);
}

template <int BM, int BN, int WM, int WN>
int32_t launch_mfma_out(const GemmPlan& plan, int max_m, int max_n, hipStream_t st) {
    if (plan.out_dtype == SBP_F32) {
        if (plan.epilogue == SBP_EPI_GELU) return launch_mfma_layout<BM, BN, WM, WN, SBP_EPI_GELU, float>(plan, max_m, max_n, st);
        return launch_mfma_layout<BM, BN, WM, WN, SBP_EPI_NONE, float>(plan, max_m, max_n, st);
    }
    if (plan.epilogue == SBP_EPI_GELU) return launch_mfma_layout<BM, BN, WM, WN, SBP_EPI_GELU, uint16_t>(plan, max_m, max_n, st);
    return launch_mfma_layout<BM, BN, WM, WN, SBP_EPI_NONE, uint16_t>(plan, max_m, max_n, st);
}

template <bool IN_BF16, typename OutT>
void launch_generic_epi(const GemmPlan& plan, dim3 grid, hipStream_t st) {
    if (plan.epilogue == SBP_EPI_GELU)
        hipLaunchKernelGGL((gemm_generic_kernel<IN_BF16, OutT, SBP_EPI_GELU>), grid, dim3(16, 16), 0, st, plan);
    else
        hipLaunchKernelGGL((gemm_generic_kernel<IN_BF16, OutT, SBP_EPI_NONE>), grid, dim3(16, 16), 0, st, plan);
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
    }
    return true;
}

}  // namespace

int32_t launch_gemm(const GemmPlan& plan, int32_t variant, hipStream_t stream) {
    int max_m = 0, max_n = 0;
    for (int g = 0; g < plan.groups; ++g) {
        if (plan.s[g].m == 0 || plan.s[g].n == 0) continue;
        max_m = plan.s[g].m > max_m ? plan.s[g].m : max_m;
        max_n = plan.s[g].n > max_n ? plan.s[g].n : max_n;
    }
    if (max_m == 0 || max_n == 0) return SBP_OK;   // every local product is empty

    const bool fast = mfma_ok(plan);
    if (variant == 1 || !fast) {
        if (variant > 1) return SBP_ERR_UNSUPPORTED;   // a forced MFMA variant cannot take this shape
        const dim3 grid((max_n + 15) / 16, (max_m + 15) / 16, plan.groups);
        if (grid.y > 65535 || grid.z > 65535) return SBP_ERR_UNSUPPORTED;
        if (plan.in_dtype == SBP_BF16) {
            if (plan.out_dtype == SBP_F32) launch_generic_epi<true, float>(plan, grid, stream);
            else launch_generic_epi<true, uint16_t>(plan, grid, stream);
        } else {
            if (plan.out_dtype != SBP_F32) return SBP_ERR_DTYPE;
            launch_generic_epi<false, float>(plan, grid, stream);
        }
        return hipGetLastError() == hipSuccess ? SBP_OK : SBP_ERR_LAUNCH;
    }
    switch (variant) {
        case 0:
        case 2: return launch_mfma_out<256, 256, 2, 2>(plan, max_m, max_n, stream);
        case 3: return launch_mfma_out<256, 256, 2, 4>(plan, max_m, max_n, stream);
        case 4: return launch_mfma_out<128, 128, 2, 2>(plan, max_m, max_n, stream);
        default: return SBP_ERR_UNSUPPORTED;
    }
}

}  // namespace sbp
