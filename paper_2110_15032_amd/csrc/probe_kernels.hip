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
//   mode 6  as mode 4 (12 reads) plus the GEMM's operand stream: every wave brings 4 KB per round from global memory
//           straight into LDS (32 KB per compute unit and round, its own 32 KB of `scratch`, so the loads hit in L2
//           after the first round): what the path L2 -> LDS costs on top
//   mode 7  as mode 6 with one of every wave's four loads taken from a 1 GiB region walked so that it misses every
//           cache (8 KB per compute unit and round from HBM: about what the GEMMs of the MLP block fetch)
//   mode 8  as mode 7 plus 4 KB per compute unit and round of streaming stores over a 512 MiB region (about what the
//           fp32 partials of GEMM2 write)
// zero != 0 fills the fragments with zeros instead of pseudo-random bf16 values of magnitude 1: same instructions,
// no operand toggling; the chip's power management then grants a higher clock.
#include <atomic>
#include <cstdio>

#include "sbp_internal.h"

namespace sbp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_SLOTS = 6144;   // 16-byte fragments per lane-row in LDS: 96 KB

typedef float f32x16 __attribute__((ext_vector_type(16)));

typedef __attribute__((address_space(1))) char gbl_char;

template <int MODE, int NRD = 16, int STREAM = 0>
__global__ __launch_bounds__(512) void probe_mfma_kernel(unsigned long long* cycles, float* sink, int iters, int zero, char* operands) {
    __shared__ bf16x8 lds[PROBE_SLOTS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // STREAM: this workgroup's 32 KB of operands (filled here, read back round after round into the upper 32 KB of LDS,
    // which nothing reads)
    [[maybe_unused]] gbl_char* mine = nullptr;
    [[maybe_unused]] uint32_t lds_dst = 0;
    [[maybe_unused]] int wv_stream = 0;
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    if constexpr (STREAM > 0) {
        char* region = operands + (size_t)blockIdx.x * 32768;
        for (int i = threadIdx.x; i < 2048; i += 512) {
            u32x4 w;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t h = (uint32_t)(i * 4 + d) * 2654435761u + 0x85EBCA6Bu * (blockIdx.x + 7);
                h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
                w[d] = zero ? 0u : ((h & 0x807F807Fu) | 0x3F803F80u);
            }
            reinterpret_cast<u32x4*>(region)[i] = w;
        }
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0): the fill is in L2 before it is read back
        const int wv = __builtin_amdgcn_readfirstlane(wave);   // uniform: the load takes a scalar base
        wv_stream = wv;
        mine = (gbl_char*)(region + wv * 4096);
        lds_dst = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)((char*)lds + 65536 + wv * 4096);
    }
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
            if constexpr (STREAM > 0) {
                // four 1 KB loads per wave, global -> LDS, lane i's 16 bytes to base + 16 i; the previous round's
                // memory operations may still be in flight
                constexpr int NHIT = STREAM >= 2 ? 3 : 4;
#pragma unroll
                for (int q = 0; q < NHIT; ++q)
                    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                                 : : "v"((uint32_t)(lane * 16 + q * 1024)), "s"(mine), "s"(lds_dst + q * 1024) : "memory", "m0");
                if constexpr (STREAM >= 2) {
                    // slot of this workgroup and round in the far regions: 131072 slots, every one touched again only
                    // after the whole region has passed through the caches
                    const uint32_t slot = (blockIdx.x * 8191u + (uint32_t)it) & 131071u;
                    gbl_char* far = (gbl_char*)(operands + (15u << 20) + (size_t)slot * 8192 + wv_stream * 1024);
                    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                                 : : "v"((uint32_t)(lane * 16)), "s"(far), "s"(lds_dst + 3 * 1024) : "memory", "m0");
                    if constexpr (STREAM >= 3) {
                        gbl_char* out = (gbl_char*)(operands + (15u << 20) + ((size_t)1 << 30) + (size_t)slot * 4096 + wv_stream * 512);
                        const u32x2 v = {(uint32_t)it, (uint32_t)lane};
                        asm volatile("global_store_dwordx2 %0, %1, %2 nt" : : "v"((uint32_t)(lane * 8)), "v"(v), "s"(out) : "memory");
                    }
                }
                __builtin_amdgcn_s_waitcnt(STREAM >= 3 ? 0x0F75 : 0x0F74);   // vmcnt(5 / 4): one round in flight
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
    if constexpr (STREAM > 0) __builtin_amdgcn_s_waitcnt(0x0070);   // the last loads land before LDS is released
    sink[blockIdx.x * 512 + threadIdx.x] = s;                   // keeps the matrix instructions alive
    if (blockIdx.x == 0 && lane == 0) cycles[wave] = t1 - t0;
}

}  // namespace

// Staging memory of sbp_probe_mfma_static (mode 6: 32 KB of operands per workgroup), held by every device the
// library runs on until the process ends.  In host code this name is only a handle for hipGetSymbolAddress:
// the device address it yields (per device) is what the kernels are given.
constexpr size_t PROBE_STATIC_BYTES = (size_t)15 << 20;
}  // namespace sbp
static __device__ __align__(256) unsigned char scratch[sbp::PROBE_STATIC_BYTES];
namespace sbp {

namespace {
// cycles: 8 uint64; sink: one float per thread of the grid; operands: staging of the modes 6-8 (see the kernel)
int32_t launch_probe(int32_t mode, int32_t iters, int32_t zero, unsigned long long* cycles, float* sink, char* operands, int grid, hipStream_t st) {
    if (mode == 0) hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else if (mode == 1) hipLaunchKernelGGL(probe_mfma_kernel<1>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else if (mode == 2) hipLaunchKernelGGL(probe_mfma_kernel<2>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else if (mode == 3) hipLaunchKernelGGL(probe_mfma_kernel<3>, dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else if (mode == 4) hipLaunchKernelGGL((probe_mfma_kernel<2, 12>), dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else if (mode == 5) hipLaunchKernelGGL((probe_mfma_kernel<2, 8>), dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else if (mode == 6) hipLaunchKernelGGL((probe_mfma_kernel<2, 12, 1>), dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else if (mode == 7) hipLaunchKernelGGL((probe_mfma_kernel<2, 12, 2>), dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    else hipLaunchKernelGGL((probe_mfma_kernel<2, 12, 3>), dim3(grid), dim3(512), 0, st, cycles, sink, iters, zero, operands);
    return launch_status(__func__);
}
}  // namespace

int32_t launch_probe_mfma(int32_t mode, int32_t iters, int32_t zero, void* scratch_arg, hipStream_t st) {
    const int grid = compute_units();
    unsigned long long* cycles = static_cast<unsigned long long*>(scratch_arg);
    float* sink = reinterpret_cast<float*>(static_cast<char*>(scratch_arg) + 64);
    // modes 6-8: 32 KB per workgroup behind the first MiB (15 MiB hold 480 such regions), then (modes 7, 8) 1 GiB that
    // is only read and 512 MiB that are only written
    char* operands = static_cast<char*>(scratch_arg) + (1 << 20);
    if (mode >= 6 && grid > 480) return SBP_ERR_UNSUPPORTED;
    return launch_probe(mode, iters, zero, cycles, sink, operands, grid, st);
}

// The same kernels with the staging memory in the library's own static device array: nothing is allocated, here
// or in the runtime calls made (the address of the array is asked of the runtime once per device and kept).
int32_t launch_probe_mfma_static(int32_t mode, int32_t iters, int32_t zero, void* out, hipStream_t st) {
    constexpr int MAX_DEV = 64;
    static std::atomic<char*> base[MAX_DEV];   // device address of `scratch` on every device, null = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return SBP_ERR_LAUNCH;
    char* ptr = base[dev].load(std::memory_order_acquire);
    if (!ptr) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // of the current device's copy
        if (e != hipSuccess || !p) {
            fprintf(stderr, "libsbp_mi355x: hipGetSymbolAddress(scratch) failed: %s\n", hipGetErrorString(e));
            return SBP_ERR_LAUNCH;
        }
        ptr = static_cast<char*>(p);
        base[dev].store(ptr, std::memory_order_release);   // two threads racing here store the same address
    }
    const int grid = compute_units();
    // mode 6 stages 32 KB per workgroup; more workgroups than the array holds are refused, never truncated
    if ((size_t)grid * 32768 > PROBE_STATIC_BYTES || (size_t)grid * 512 * sizeof(float) + 64 > ((size_t)1 << 20)) return SBP_ERR_UNSUPPORTED;
    unsigned long long* cycles = static_cast<unsigned long long*>(out);
    float* sink = reinterpret_cast<float*>(static_cast<char*>(out) + 64);
    return launch_probe(mode, iters, zero, cycles, sink, ptr, grid, st);
}

}  // namespace sbp
