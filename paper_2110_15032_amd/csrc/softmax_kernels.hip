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

// SUMEXP: m is passed as -max * log2(e), so that exp(v - max) is one FMA and one hardware exp2
// (relative error about |v - max| * 1e-7: the argument is at most 0 and a term below 2^-126 adds
// nothing to a sum that contains exp(0) = 1 somewhere on the row's devices)
constexpr float LOG2E = 1.4426950408889634f;
template <bool SUMEXP>
__device__ inline float fold(float acc, float v, float m) {
    if constexpr (SUMEXP) return acc + __builtin_amdgcn_exp2f(fmaf(v, LOG2E, m));
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
    const float m = SUMEXP ? -p.gmax[shard][row] * LOG2E : 0.0f;
    float acc = ident;
    if (cols > 0) {
        constexpr int EPV = BF16 ? 8 : 4;  // elements per 16-byte vector
        const char* base = static_cast<const char*>(p.logits[shard]) + (int64_t)row * p.ld[shard] * (BF16 ? 2 : 4);
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

// ------------------------------------------------------------------------------------------------
// Sparse cross entropy on the same S(1) logits (Sec. 6.3.1): with the global row max m and
// denominator s in hand (B), the loss needs one logit per row, held by exactly one device, so every
// device writes a partial vector (P(sum)); the gradient is elementwise on every shard.
// ------------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(RS_THREADS) void xent_loss_kernel(XentPlan p) {
    const int i = blockIdx.y;
    const int64_t r = (int64_t)blockIdx.x * RS_THREADS + threadIdx.x;
    if (r >= p.rows) return;
    const int32_t c = p.labels[i][r] - p.begin[i];
    float out = 0.0f;
    if (c >= 0 && c < p.cols[i]) {
        const int64_t pos = r * p.ld[i] + c;
        float l;
        if constexpr (BF16) l = __uint_as_float((uint32_t) static_cast<const uint16_t*>(p.logits[i])[pos] << 16);
        else l = static_cast<const float*>(p.logits[i])[pos];
        out = logf(p.denom[i][r]) + p.gmax[i][r] - l;
    }
    static_cast<float*>(p.out[i])[r] = out;
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf16(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// VE elements per lane: 8 bf16 / 4 fp32 (16 bytes) when the row pitch allows, else 1
template <bool BF16, int VE>
__global__ __launch_bounds__(RS_THREADS) void xent_grad_kernel(XentPlan p) {
    const int i = blockIdx.y;
    const uint32_t cols_v = (uint32_t)p.cols[i] / VE;
    if (cols_v == 0) return;
    // (row, vector) of this lane's first item by one division, then advanced by the grid stride with adds only:
    // a 64-bit division per item costs more vector instructions than the item's arithmetic and made the kernel
    // instruction-bound instead of memory-bound
    const uint64_t stride = (uint64_t)gridDim.x * RS_THREADS;
    const uint32_t dr = (uint32_t)(stride / cols_v), dc = (uint32_t)(stride % cols_v);
    const uint64_t first = (uint64_t)blockIdx.x * RS_THREADS + threadIdx.x;
    uint64_t r64 = first / cols_v;
    uint32_t cv = (uint32_t)(first % cols_v);
    for (; r64 < (uint64_t)p.rows; r64 += dr, cv += dc) {
        if (cv >= cols_v) {
            cv -= cols_v;
            if (++r64 >= (uint64_t)p.rows) break;
        }
        const uint32_t r = (uint32_t)r64;
        const uint32_t c = cv * VE;
        const int32_t y = p.labels[i][r];
        const bool live = y >= 0 && y < p.total_cols;
        const float g = live ? p.grad[i][r] : 0.0f;
        const float m = p.gmax[i][r], inv = 1.0f / p.denom[i][r];
        const int32_t yc = y - p.begin[i] - (int32_t)c;   // position of the label inside this group, if any
        const int64_t pos = (int64_t)r * p.ld[i] + c, opos = (int64_t)r * p.ld_out[i] + c;
        float v[VE];
        if constexpr (BF16 && VE == 8) {
            // streaming load: the gradient pass is the last reader of the logits (measured 2 % faster than a cached load;
            // two items per lane and round, both loaded before either is worked on, 1 % slower than this)
            const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.logits[i]) + pos));
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                v[2 * d] = bf16_lo(w[d]);
                v[2 * d + 1] = bf16_hi(w[d]);
            }
        } else if constexpr (!BF16 && VE == 4) {
            const f32x4 w = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(static_cast<const float*>(p.logits[i]) + pos));
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = w[e];
        } else {
            if constexpr (BF16) v[0] = __uint_as_float((uint32_t) static_cast<const uint16_t*>(p.logits[i])[pos] << 16);
            else v[0] = static_cast<const float*>(p.logits[i])[pos];
        }
#pragma unroll
        for (int e = 0; e < VE; ++e) v[e] = (__expf(v[e] - m) * inv - (e == yc ? 1.0f : 0.0f)) * g;
        if constexpr (BF16 && VE == 8) {
            const u32x4 o = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(static_cast<uint16_t*>(p.out[i]) + opos));
        } else if constexpr (!BF16 && VE == 4) {
            const f32x4 o = {v[0], v[1], v[2], v[3]};
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(static_cast<float*>(p.out[i]) + opos));
        } else {
            if constexpr (BF16) static_cast<uint16_t*>(p.out[i])[opos] = (uint16_t)(pack_bf16(v[0], 0.0f) & 0xFFFFu);
            else static_cast<float*>(p.out[i])[opos] = v[0];
        }
    }
}

}  // namespace

int32_t launch_xent_loss(const XentPlan& plan, hipStream_t stream) {
    if (plan.rows == 0) return SBP_OK;
    const int64_t bx = (plan.rows + RS_THREADS - 1) / RS_THREADS;
    if (bx > 0x7FFFFFFF) return SBP_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)bx, (uint32_t)plan.k);
    if (plan.dtype == SBP_BF16) hipLaunchKernelGGL(xent_loss_kernel<true>, grid, dim3(RS_THREADS), 0, stream, plan);
    else hipLaunchKernelGGL(xent_loss_kernel<false>, grid, dim3(RS_THREADS), 0, stream, plan);
    return launch_status(__func__);
}

int32_t launch_xent_grad(const XentPlan& plan, hipStream_t stream) {
    if (plan.rows == 0 || plan.total_cols == 0) return SBP_OK;
    const bool bf = plan.dtype == SBP_BF16;
    const int epv = bf ? 8 : 4;
    bool vec = true;
    int64_t max_units = 0;
    for (int i = 0; i < plan.k; ++i) {
        if (plan.cols[i] % epv || plan.ld[i] % epv || plan.ld_out[i] % epv) vec = false;
        max_units = plan.cols[i] > max_units ? plan.cols[i] : max_units;
    }
    max_units = max_units * plan.rows / (vec ? epv : 1);
    int64_t bx = (max_units + RS_THREADS - 1) / RS_THREADS;
    // at most 65536 workgroups, grid-stride beyond (2 GB of bf16 logits: 0.68 ms; with one vector per lane and
    // half a million short-lived workgroups 0.74 ms, with 16384 workgroups 0.73 ms)
    const int64_t cap = (1 << 16) / plan.k;
    if (bx > cap) bx = cap;
    if (bx < 1) bx = 1;
    const dim3 grid((uint32_t)bx, (uint32_t)plan.k);
    if (bf && vec) hipLaunchKernelGGL((xent_grad_kernel<true, 8>), grid, dim3(RS_THREADS), 0, stream, plan);
    else if (bf) hipLaunchKernelGGL((xent_grad_kernel<true, 1>), grid, dim3(RS_THREADS), 0, stream, plan);
    else if (vec) hipLaunchKernelGGL((xent_grad_kernel<false, 4>), grid, dim3(RS_THREADS), 0, stream, plan);
    else hipLaunchKernelGGL((xent_grad_kernel<false, 1>), grid, dim3(RS_THREADS), 0, stream, plan);
    return launch_status(__func__);
}

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
