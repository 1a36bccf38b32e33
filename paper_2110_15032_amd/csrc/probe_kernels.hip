// Diagnostic kernels behind sbp_probe_mfma: what the matrix pipes of this chip sustain, and what operand
// fragment reads between the matrix instructions cost, measured in isolation.  They put the rate of the
// GEMM kernels (gemm_kernels.hip, gemm_pingpong_kernel.hip) into context; nothing of the SBP method runs here.
//
// One workgroup of 8 waves per compute unit (two waves per SIMD, as in the GEMM kernels; 96 KB of LDS keep a
// second workgroup off the unit).  Every wave owns 16 accumulator blocks of v_mfma_f32_16x16x32_bf16 and
// runs `iters` rounds of 32 matrix instructions on 4 + 4 operand fragments:
//   mode 0  matrix instructions only, no synchronisation
//   mode 1  lockstep: both waves of a SIMD interleave 16 fragment reads (ds_read_b128) with their 32 matrix
//           instructions, one workgroup barrier per round      (the schedule of gemm_mfma_persist16_kernel)
//   mode 2  ping-pong: the waves 4-7 run one phase behind the waves 0-3; a wave alternates between reading its
//           16 fragments and issuing its 32 matrix instructions, a barrier between phases
//                                                              (the schedule of gemm_pingpong_kernel)
//   mode 3  as mode 0 with v_mfma_f32_32x32x16_bf16 (16 instructions of twice the work per round)
//   mode 4, 5  as mode 2 with 12 and with 8 fragment reads per round: what the fragment traffic costs
// zero != 0 fills the fragments with zeros instead of pseudo-random bf16 values of magnitude 1: same instructions,
// no operand toggling; the chip's power management then grants a higher clock.
#include "sbp_internal.h"

namespace sbp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_SLOTS = 6144;   // 16-byte fragments per lane-row in LDS: 96 KB

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int MODE, int NRD = 16>
__global__ __launch_bounds__(512) void probe_mfma_kernel(unsigned long long* cycles, float* sink, int iters, int zero) {
    __shared__ bf16x8 lds[PROBE_SLOTS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < PROBE_SLOTS; i += 512) {
        u32x4 w;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t h = (uint32_t)(i * 4 + d) * 2654435761u + 0x9E3779B9u * (blockIdx.x + 1);
            h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
            // two bf16 values with exponent of 1.0, random sign and mantissa
            w[d] = zero ? 0u : ((h & 0x807F807Fu) | 0x3F803F80u);
        }
        lds[i] = __builtin_bit_cast(bf16x8, w);
    }
    __syncthreads();
    f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = f32x4{0, 0, 0, 0};
    bf16x8 fa[2][4], fb[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[s][i] = lds[lane + 64 * (i + 8 * s)];
            fb[s][i] = lds[lane + 64 * (i + 4 + 8 * s)];
        }
    __syncthreads();
    if (MODE == 2 && wave >= 4) __builtin_amdgcn_s_barrier();   // the second group runs one phase behind
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
        if constexpr (MODE == 3) {
            // the 16 accumulator blocks of 16x16 regrouped as 4 blocks of 32x32
            f32x16* big = reinterpret_cast<f32x16*>(acc);
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int q = 0; q < 8; ++q) big[q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[g][q & 3], fa[g][q >> 1], big[q & 3], 0, 0, 0);
        } else if constexpr (MODE == 0) {
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[g][q & 3], fa[g][q >> 2], acc[q], 0, 0, 0);
        } else if constexpr (MODE == 1) {
            // half g multiplies the fragments of slot g while those of the other slot are read behind the first eight
            // matrix instructions (one read each, pinned in place)
#pragma unroll
            for (int g = 0; g < 2; ++g) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[g][q & 3], fa[g][q >> 2], acc[q], 0, 0, 0);
                    if (q < 4) fa[g ^ 1][q] = lds[lane + 64 * ((q + it + 16 * g) & 63)];
                    else if (q < 8) fb[g ^ 1][q - 4] = lds[lane + 64 * ((q + it + 7 + 16 * g) & 63)];
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_s_barrier();
        } else {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (8 * s + i < NRD) fa[s][i] = lds[lane + 64 * ((i + it + 16 * s) & 63)];
                    if (8 * s + 4 + i < NRD) fb[s][i] = lds[lane + 64 * ((i + it + 7 + 16 * s) & 63)];
                }
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[g][q & 3], fa[g][q >> 2], acc[q], 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
        }
    }
    const unsigned long long t1 = __builtin_readcyclecounter();
    if (MODE == 2 && wave < 4) __builtin_amdgcn_s_barrier();    // pairs with the last barrier of the second group
    float s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    sink[blockIdx.x * 512 + threadIdx.x] = s;                   // keeps the matrix instructions alive
    if (blockIdx.x == 0 && lane == 0) cycles[wave] = t1 - t0;
}

}  // namespace

int32_t launch_probe_mfma(int32_t mode, int32_t iters, int32_t zero, void* scratch, hipStream_t st) {
    const int grid = compute_units();
    unsigned long long* cycles = static_cast<unsigned long long*>(scratch);
    float* sink = reinterpret_cast<float*>(static_cast<char*>(scratch) + 64);
    if (mode == 0) hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero);
    else if (mode == 1) hipLaunchKernelGGL(probe_mfma_kernel<1>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero);
    else if (mode == 2) hipLaunchKernelGGL(probe_mfma_kernel<2>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero);
    else if (mode == 3) hipLaunchKernelGGL(probe_mfma_kernel<3>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero);
    else if (mode == 4) hipLaunchKernelGGL((probe_mfma_kernel<2, 12>), dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero);
    else hipLaunchKernelGGL((probe_mfma_kernel<2, 8>), dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero);
    return launch_status(__func__);
}

}  // namespace sbp
