// Local row reductions of the model-parallel softmax (paper Sec. 6.3.1): each device reduces the
// columns of the logits it holds, first to a row max (P(max)), then -- once the max has been boxed
// to B -- to a row sum of exp(l - max) (P(sum)).  One workgroup per (row, shard); 16-byte loads
// where the row pitch allows, wavefront shuffles then one LDS hop across the four waves.
#include "sbp_internal.h"

namespace sbp {
namespace {

constexpr int RS_THREADS = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <bool SUMEXP>
__device__ inline float fold(float acc, float v, float m) {
    if constexpr (SUMEXP) return acc + expf(v - m);
    else return fmaxf(acc, v);
}

template <bool SUMEXP>
__device__ inline float wave_reduce(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(v, off, 64);
        v = SUMEXP ? v + o : fmaxf(v, o);
    }
    return v;
}

template <bool SUMEXP, bool BF16>
__global__ __launch_bounds__(RS_THREADS) void row_stat_kernel(RowStatPlan p) {
    const int shard = blockIdx.y;
    const int64_t row = blockIdx.x;
    const int32_t cols = p.cols[shard];
    const float ident = SUMEXP ? 0.0f : -INFINITY;
    const float m = SUMEXP ? p.gmax[shard][row] : 0.0f;
    float acc = ident;
    if (cols > 0) {
        constexpr int EPV = BF16 ? 8 : 4;  // elements per 16-byte vector
        const char* base = static_cast<const char*>(p.logits[shard]) + (int64_t)row * cols * (BF16 ? 2 : 4);
        // rows start 16-byte aligned only when the pitch is a multiple of EPV; otherwise peel
        const int32_t mis = (int32_t)((reinterpret_cast<uintptr_t>(base) & 15u) / (BF16 ? 2 : 4));
        int32_t head = mis ? EPV - mis : 0;
        if (head > cols) head = cols;
        const int32_t nvec = (cols - head) / EPV;
        const int32_t tail0 = head + nvec * EPV;
        auto elem = [&](int32_t c) -> float {
            if constexpr (BF16) return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(base)[c] << 16);
            else return reinterpret_cast<const float*>(base)[c];
        };
        for (int32_t c = threadIdx.x; c < head; c += RS_THREADS) acc = fold<SUMEXP>(acc, elem(c), m);
        for (int32_t c = tail0 + threadIdx.x; c < cols; c += RS_THREADS) acc = fold<SUMEXP>(acc, elem(c), m);
        const char* vbase = base + (int64_t)head * (BF16 ? 2 : 4);
        float a0 = ident, a1 = ident, a2 = ident, a3 = ident;   // four chains per lane
        for (int32_t v = threadIdx.x; v < nvec; v += RS_THREADS) {
            if constexpr (BF16) {
                const u32x4 w = reinterpret_cast<const u32x4*>(vbase)[v];
                a0 = fold<SUMEXP>(fold<SUMEXP>(a0, bf16_lo(w.x), m), bf16_hi(w.x), m);
                a1 = fold<SUMEXP>(fold<SUMEXP>(a1, bf16_lo(w.y), m), bf16_hi(w.y), m);
                a2 = fold<SUMEXP>(fold<SUMEXP>(a2, bf16_lo(w.z), m), bf16_hi(w.z), m);
                a3 = fold<SUMEXP>(fold<SUMEXP>(a3, bf16_lo(w.w), m), bf16_hi(w.w), m);
            } else {
                const f32x4 w = reinterpret_cast<const f32x4*>(vbase)[v];
                a0 = fold<SUMEXP>(a0, w.x, m);
                a1 = fold<SUMEXP>(a1, w.y, m);
                a2 = fold<SUMEXP>(a2, w.z, m);
                a3 = fold<SUMEXP>(a3, w.w, m);
            }
        }
        if constexpr (SUMEXP) acc += (a0 + a1) + (a2 + a3);
        else acc = fmaxf(fmaxf(acc, fmaxf(a0, a1)), fmaxf(a2, a3));
    }
    acc = wave_reduce<SUMEXP>(acc);
    __shared__ float part[RS_THREADS / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = part[0];
#pragma unroll
        for (int w = 1; w < RS_THREADS / 64; ++w) r = SUMEXP ? r + part[w] : fmaxf(r, part[w]);
        p.out[shard][row] = r;
    }
}

}  // namespace

int32_t launch_row_stat(const RowStatPlan& plan, bool sumexp, hipStream_t stream) {
    if (plan.rows == 0) return SBP_OK;
    if (plan.rows > 0x7FFFFFFF) return SBP_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)plan.rows, (uint32_t)plan.k);
    const dim3 block(RS_THREADS);
    const bool bf = plan.dtype == SBP_BF16;
    if (sumexp) {
        if (bf) hipLaunchKernelGGL((row_stat_kernel<true, true>), grid, block, 0, stream, plan);
        else hipLaunchKernelGGL((row_stat_kernel<true, false>), grid, block, 0, stream, plan);
    } else {
        if (bf) hipLaunchKernelGGL((row_stat_kernel<false, true>), grid, block, 0, stream, plan);
        else hipLaunchKernelGGL((row_stat_kernel<false, false>), grid, block, 0, stream, plan);
    }
    return launch_status(__func__);
}

}  // namespace sbp
