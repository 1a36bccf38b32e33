// Boxing kernels (paper Sec. 3.2, Table 2), for shard buffers in one HBM: ki input devices, ko output
// devices.  On one device set ki = ko = k (the table's "same" column); between disjoint placements
// the two counts are independent (its "disjoint" column) and the task lists below generalise as
// noted at make_task.
//
// Every conversion is a set of rectangle tasks (blockIdx.y = task).  A task reads one rows x cols
// rectangle from NS source shards that all use the same offset and pitch, combines them in shard
// order (copy / fp32 sum / fp32 max) and writes the result into ND destination shards that all use
// the same offset and pitch.  The rectangles follow from the balanced split alone, so the kernel
// derives them from (mode, task id) and needs no task table in memory:
//
//   P -> B        1 task : all k sources, all k destinations, whole tensor       (all-reduce)
//   P -> S(a)     k tasks: all k sources at slice j        -> out_j              (reduce-scatter)
//   S(a) -> B     k tasks: in_i                            -> slice i of all k   (all-gather; 16-byte
//                          vectors take box_gather_bcast_kernel instead, see there)
//   S(a) -> S(b)  k*k    : in_i restricted to slice j of b -> out_j at slice i   (all2all)
//   B -> S(a)     k tasks: slice j of in_j (its own copy)  -> out_j              (local slice)
//   X -> X        k tasks: in_i -> out_i                                         (identity)
//   S(a), B -> P  own kernels (box_to_partial*_kernel): own values kept, identity elsewhere
//   ki != ko only: S(a) -> S(a) takes the all2all task list (ki*ko range intersections), B -> B is the
//                  all-gather of a tensor "split" over one device, and
//   P -> P        ko tasks: partials j, j + ko, j + 2 ko, ... combined in that order -> out_j
//
// HBM-bound: every input byte is read once and every output byte written once, with the widest
// vector (up to 16 B per lane) that all offsets and pitches of the conversion allow.
#include <atomic>
#include <cstdlib>

#include "sbp_internal.h"

namespace sbp {
namespace {

enum BoxMode : int32_t { M_P2B = 0, M_P2S, M_S2B, M_S2S, M_B2S, M_IDENT, M_P2P };

struct BoxParams {
    const void* src[SBP_MAX_K];
    void* dst[SBP_MAX_K];
    int64_t rows, cols;   // global shape in elements
    int32_t ki, ko;       // input / output device count
    int32_t mode;
    int32_t axis_in;      // split axis of the input  (S inputs), else -1
    int32_t axis_out;     // split axis of the output (S outputs), else -1
    int32_t vec_elems;    // elements per vector access
    int32_t sbp_same;     // M_IDENT: signature (decides the local shape)
    // M_S2S with both sides split along the SAME axis (ki != ko): only ki + ko - 1 of the ki * ko
    // (input, output) pairs overlap at most; the launcher lists them here so that no workgroup is
    // started for an empty pair (npairs == 0: task t is pair (t / ko, t % ko))
    int32_t npairs;
    uint8_t pair_i[2 * SBP_MAX_K], pair_j[2 * SBP_MAX_K];
    // reductions only: blockIdx.z = conversion b of a batch, its sources src[b * ki + i], its destinations dst[b * ko + j]
    int32_t batch;
};

struct Task {
    int32_t s0, ns;       // sources  s0, s0 + sstep, ... (ns of them)
    int32_t d0, nd;       // destinations [d0, d0 + nd)
    int64_t src_off, dst_off, src_ld, dst_ld;   // elements
    int64_t rows, cols;   // rectangle, elements
    int32_t sstep;        // distance between consecutive sources (1 except P -> P)
};

__host__ __device__ inline void range_of(int64_t n, int32_t k, int32_t i, int32_t axis_is_split, int64_t& b, int64_t& l) {
    if (axis_is_split) {
        b = split_begin(n, k, i);
        l = split_len(n, k, i);
    } else {
        b = 0;
        l = n;
    }
}

// Geometry of task t.  Shared by the launcher (alignment analysis, grid sizing) and the kernel.
__host__ __device__ inline Task make_task(const BoxParams& p, int32_t t) {
    Task T{};
    const int32_t ki = p.ki, ko = p.ko;
    int64_t rb, rl, cb, cl;
    switch (p.mode) {
        case M_P2B:
            T = {0, ki, 0, ko, 0, 0, p.cols, p.cols, p.rows, p.cols};
            break;
        case M_P2S: {
            range_of(p.rows, ko, t, p.axis_out == 0, rb, rl);
            range_of(p.cols, ko, t, p.axis_out == 1, cb, cl);
            T = {0, ki, t, 1, rb * p.cols + cb, 0, p.cols, cl, rl, cl};
            break;
        }
        case M_S2B: {
            range_of(p.rows, ki, t, p.axis_in == 0, rb, rl);
            range_of(p.cols, ki, t, p.axis_in == 1, cb, cl);
            T = {t, 1, 0, ko, 0, rb * p.cols + cb, cl, p.cols, rl, cl};
            break;
        }
        case M_S2S: {
            const int32_t i = p.npairs ? p.pair_i[t] : t / ko, j = p.npairs ? p.pair_j[t] : t % ko;   // in_i -> out_j
            int64_t irb, irl, icb, icl, orb, orl, ocb, ocl;
            range_of(p.rows, ki, i, p.axis_in == 0, irb, irl);
            range_of(p.cols, ki, i, p.axis_in == 1, icb, icl);
            range_of(p.rows, ko, j, p.axis_out == 0, orb, orl);
            range_of(p.cols, ko, j, p.axis_out == 1, ocb, ocl);
            // intersection in global coordinates (empty for most pairs when both sides split the same axis)
            const int64_t r0 = irb > orb ? irb : orb, r1 = (irb + irl) < (orb + orl) ? (irb + irl) : (orb + orl);
            const int64_t c0 = icb > ocb ? icb : ocb, c1 = (icb + icl) < (ocb + ocl) ? (icb + icl) : (ocb + ocl);
            T = {i, 1, j, 1, (r0 - irb) * icl + (c0 - icb), (r0 - orb) * ocl + (c0 - ocb), icl, ocl,
                 r1 > r0 ? r1 - r0 : 0, c1 > c0 ? c1 - c0 : 0};
            break;
        }
        case M_B2S: {   // device t takes its slice from a copy on "its" input device (its own when ki == ko)
            range_of(p.rows, ko, t, p.axis_out == 0, rb, rl);
            range_of(p.cols, ko, t, p.axis_out == 1, cb, cl);
            T = {t % ki, 1, t, 1, rb * p.cols + cb, 0, p.cols, cl, rl, cl};
            break;
        }
        case M_P2P: {   // partials t, t + ko, ... -> out_t; none when t >= ki (the kernel then writes the identity)
            T = {t, t < ki ? (ki - t + ko - 1) / ko : 0, t, 1, 0, 0, p.cols, p.cols, p.rows, p.cols};
            break;
        }
        default: {  // M_IDENT (ki == ko)
            range_of(p.rows, ki, t, p.sbp_same == 0, rb, rl);
            range_of(p.cols, ki, t, p.sbp_same == 1, cb, cl);
            T = {t, 1, t, 1, 0, 0, cl, cl, rl, cl};
            break;
        }
    }
    T.sstep = p.mode == M_P2P ? ko : 1;
    // A rectangle as wide as both pitches is one contiguous run: flatten it so the kernel's
    // row / column split degenerates (no division on the hot path).
    if (T.cols == T.src_ld && T.cols == T.dst_ld) {
        T.cols = T.rows * T.cols;
        T.rows = T.cols ? 1 : 0;
        T.src_ld = T.dst_ld = T.cols;
    }
    return T;
}

// native clang vectors: one global_load / global_store of 4, 8 or 16 bytes per lane
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int OP, typename V>
__device__ inline V combine(V a, V b) {
    if constexpr (OP == BOX_SUM) return a + b;
    else return __builtin_elementwise_max(a, b);
}

constexpr int BOX_THREADS = 256;

// Reduction tasks: NS sources (compile-time when KS > 0), fp32 math in shard order.
template <typename V, int OP, int KS, int UNROLL>
__global__ __launch_bounds__(BOX_THREADS) void box_reduce_kernel(BoxParams p) {
    const Task T = make_task(p, blockIdx.y);
    const int32_t ns = KS > 0 ? KS : T.ns;
    const int32_t sb = (int32_t)blockIdx.z * p.ki, db = (int32_t)blockIdx.z * p.ko;   // this conversion's pointers
    const uint32_t cols_v = (uint32_t)(T.cols / p.vec_elems);
    const uint32_t total = (uint32_t)T.rows * cols_v;
    const int64_t src_ld_v = T.src_ld / p.vec_elems, dst_ld_v = T.dst_ld / p.vec_elems;
    const int64_t src_off_v = T.src_off / p.vec_elems, dst_off_v = T.dst_off / p.vec_elems;
    // a workgroup covers UNROLL consecutive runs of BOX_THREADS vectors
    const uint32_t stride = BOX_THREADS;
    for (uint32_t base = blockIdx.x * BOX_THREADS * UNROLL + threadIdx.x; base < total; base += gridDim.x * BOX_THREADS * UNROLL) {
        V acc[UNROLL];
        int64_t dpos[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t idx = base + u * stride;
            if (idx < total) {
                const uint32_t r = T.rows == 1 ? 0 : idx / cols_v;
                const uint32_t c = idx - r * cols_v;
                const int64_t spos = src_off_v + (int64_t)r * src_ld_v + c;
                dpos[u] = dst_off_v + (int64_t)r * dst_ld_v + c;
                V a;
                if constexpr (KS > 0) {   // sources 0 .. KS-1
                    a = __builtin_nontemporal_load(static_cast<const V*>(p.src[sb]) + spos);
                    V part[KS];
#pragma unroll
                    for (int i = 1; i < KS; ++i) part[i] = __builtin_nontemporal_load(static_cast<const V*>(p.src[sb + i]) + spos);
#pragma unroll
                    for (int i = 1; i < KS; ++i) a = combine<OP>(a, part[i]);
                } else {
                    if constexpr (OP == BOX_SUM) a = V(0.0f);
                    else a = V(-__builtin_inff());
                    if (ns > 0) a = __builtin_nontemporal_load(static_cast<const V*>(p.src[sb + T.s0]) + spos);
                    for (int i = 1; i < ns; ++i) {
                        const V b = __builtin_nontemporal_load(static_cast<const V*>(p.src[sb + T.s0 + i * T.sstep]) + spos);
                        a = combine<OP>(a, b);
                    }
                }
                acc[u] = a;
            }
        }
        for (int j = 0; j < T.nd; ++j) {   // destination by destination: UNROLL x 4 KB contiguous each
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t idx = base + u * stride;
                if (idx < total) __builtin_nontemporal_store(acc[u], static_cast<V*>(p.dst[db + T.d0 + j]) + dpos[u]);
            }
        }
    }
}

// The same reduction with the k source streams out of phase.  Equally sized shard buffers allocated one after
// the other put equal offsets of all k sources on the same memory channel and bank, and the plain kernel asks for
// exactly those k lines at once.  Here a lane owns KS vectors 4 KB apart and vector u takes source s - u in time
// slice s (s = 0 .. 2 KS - 2): every vector still receives its sources in shard order 0 .. KS - 1 (same sums, bit
// for bit), but the KS loads of one slice go to KS different offsets.
template <typename V, int OP, int KS>
__global__ __launch_bounds__(BOX_THREADS) void box_reduce_diag_kernel(BoxParams p) {
    const Task T = make_task(p, blockIdx.y);
    const int32_t sb = (int32_t)blockIdx.z * p.ki, db = (int32_t)blockIdx.z * p.ko;   // this conversion's pointers
    const uint32_t cols_v = (uint32_t)(T.cols / p.vec_elems);
    const uint32_t total = (uint32_t)T.rows * cols_v;
    const int64_t src_ld_v = T.src_ld / p.vec_elems, dst_ld_v = T.dst_ld / p.vec_elems;
    const int64_t src_off_v = T.src_off / p.vec_elems, dst_off_v = T.dst_off / p.vec_elems;
    for (uint32_t base = blockIdx.x * BOX_THREADS * KS + threadIdx.x; base < total; base += gridDim.x * BOX_THREADS * KS) {
        V acc[KS];
        int64_t spos[KS], dpos[KS];
#pragma unroll
        for (int u = 0; u < KS; ++u) {
            uint32_t idx = base + u * BOX_THREADS;
            idx = idx < total ? idx : total - 1;      // clamped: loaded, never stored
            const uint32_t r = T.rows == 1 ? 0 : idx / cols_v;
            const uint32_t c = idx - r * cols_v;
            spos[u] = src_off_v + (int64_t)r * src_ld_v + c;
            dpos[u] = dst_off_v + (int64_t)r * dst_ld_v + c;
        }
#pragma unroll
        for (int s = 0; s < 2 * KS - 1; ++s) {
#pragma unroll
            for (int u = 0; u < KS; ++u) {
                const int i = s - u;
                if (i < 0 || i >= KS) continue;
                const V v = __builtin_nontemporal_load(static_cast<const V*>(p.src[sb + i]) + spos[u]);
                acc[u] = i == 0 ? v : combine<OP>(acc[u], v);
            }
        }
        for (int j = 0; j < T.nd; ++j) {
#pragma unroll
            for (int u = 0; u < KS; ++u) {
                const uint32_t idx = base + u * BOX_THREADS;
                if (idx < total) __builtin_nontemporal_store(acc[u], static_cast<V*>(p.dst[db + T.d0 + j]) + dpos[u]);
            }
        }
    }
}

// Copy tasks: one source, ND destinations, raw words.
template <typename V, int UNROLL>
__global__ __launch_bounds__(BOX_THREADS) void box_copy_kernel(BoxParams p) {
    const Task T = make_task(p, blockIdx.y);
    const uint32_t cols_v = (uint32_t)(T.cols / p.vec_elems);
    const uint32_t total = (uint32_t)T.rows * cols_v;
    const int64_t src_ld_v = T.src_ld / p.vec_elems, dst_ld_v = T.dst_ld / p.vec_elems;
    const V* __restrict__ src = static_cast<const V*>(p.src[T.s0]) + T.src_off / p.vec_elems;
    const int64_t dst_off_v = T.dst_off / p.vec_elems;
    const uint32_t stride = gridDim.x * BOX_THREADS;
    for (uint32_t base = blockIdx.x * BOX_THREADS + threadIdx.x; base < total; base += stride * UNROLL) {
        V val[UNROLL];
        int64_t dpos[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t idx = base + u * stride;
            if (idx < total) {
                const uint32_t r = T.rows == 1 ? 0 : idx / cols_v;
                const uint32_t c = idx - r * cols_v;
                val[u] = __builtin_nontemporal_load(src + (int64_t)r * src_ld_v + c);
                dpos[u] = dst_off_v + (int64_t)r * dst_ld_v + c;
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t idx = base + u * stride;
            if (idx < total) {
                for (int j = 0; j < T.nd; ++j) __builtin_nontemporal_store(val[u], static_cast<V*>(p.dst[T.d0 + j]) + dpos[u]);
            }
        }
    }
}

// S(a) -> B (all-gather) at scale.  Writing every vector to all k destinations at once keeps k write
// streams open across the chip, and HBM takes that badly (measured on 16 x 1 GiB: 5.1 TB/s, against
// 6.9 TB/s for one stream).  So the logical tensor is cut into chunks of `pieces` x 4 KB and each chunk
// is written to destination 0, then 1, ... by consecutive groups of workgroups:
//     block id = (chunk * k + destination) * pieces + piece
// At any time the chip then writes one or two contiguous runs.  The chunk is read k times, but only
// the first read reaches HBM: with pieces a multiple of 8 a piece is handled by the same XCD in every
// pass, and 8 MB chunks (1 MB per XCD) stay in its L2 (plain loads; the stores stream past it).
// Sources are read-only, so the passes need no ordering among themselves.
// The index arithmetic is kept off the per-vector path where it can be (an HBM-bound kernel has
// about 80 lane-instructions per 16-byte vector to spend): block and row decomposition once per
// workgroup, the owner of a position from a float estimate with a +-1 fix-up.  Measured on
// 16 x 1 GiB: 6.3 TB/s with one vector per lane and 2048 pieces, 6.1 / 5.7 TB/s with two / four
// vectors per lane at the same chunk size, so one it is.
constexpr int BCAST_U = 1;
template <typename V>
__global__ __launch_bounds__(BOX_THREADS) void box_gather_bcast_kernel(BoxParams p, uint32_t log2_pieces, uint32_t total,
                                                                        uint32_t q, uint32_t rem) {
    __shared__ const V* sp[SBP_MAX_K];
    if ((int)threadIdx.x < p.ki) sp[threadIdx.x] = static_cast<const V*>(p.src[threadIdx.x]);
    __syncthreads();
    const uint32_t k = (uint32_t)p.ko;
    const uint32_t piece = blockIdx.x & ((1u << log2_pieces) - 1);
    const uint32_t cj = blockIdx.x >> log2_pieces;
    const uint32_t chunk = cj / k, j = cj - chunk * k;
    const uint32_t idx0 = ((chunk << log2_pieces) + piece) * (uint32_t)(BOX_THREADS * BCAST_U);   // first vector of the piece
    if (idx0 >= total) return;
    const uint32_t vec = (uint32_t)p.vec_elems, lv = __builtin_ctz(vec);
    const uint32_t cols_v = (uint32_t)(p.cols >> lv);
    const uint32_t r0 = idx0 / cols_v, c0 = idx0 - r0 * cols_v;
    // balanced split of the split axis: shards [0, rem) hold q + 1 indices, the rest q; edge = first index of the rest
    const uint32_t edge = rem * (q + 1);
    const float inv_hi = 1.0f / (float)(q + 1), inv_lo = 1.0f / (float)(q ? q : 1);
    const bool by_rows = p.axis_in == 0;
    V val[BCAST_U];
    uint32_t pos[BCAST_U];
#pragma unroll
    for (int u = 0; u < BCAST_U; ++u) {
        const uint32_t idx = idx0 + u * BOX_THREADS + threadIdx.x;
        pos[u] = idx;
        if (idx < total) {
            uint32_t c = c0 + u * BOX_THREADS + threadIdx.x, r = r0;
            if (cols_v >= (uint32_t)(BOX_THREADS * BCAST_U)) {   // a piece crosses at most one row boundary
                if (c >= cols_v) {
                    c -= cols_v;
                    ++r;
                }
            } else {
                const uint32_t w = c / cols_v;
                r += w;
                c -= w * cols_v;
            }
            const uint32_t x = by_rows ? r : c << lv;
            // owner i of index x: quotient below 64, so the float estimate is off by one at most
            uint32_t i, begin, len;
            if (x < edge) {
                i = (uint32_t)((float)x * inv_hi);
                begin = i * (q + 1);
                len = q + 1;
            } else {
                i = (uint32_t)((float)(x - edge) * inv_lo);
                begin = edge + i * q;
                i += rem;
                len = q;
            }
            if (x < begin) {
                --i;
                len = q + (i < rem ? 1u : 0u);
                begin -= len;
            } else if (x >= begin + len) {
                begin += len;
                ++i;
                len = q + (i < rem ? 1u : 0u);
            }
            const int64_t spos = by_rows ? (int64_t)(r - begin) * cols_v + c : ((int64_t)r * len + (x - begin)) >> lv;
            val[u] = sp[i][spos];
        }
    }
    V* __restrict__ dst = static_cast<V*>(p.dst[j]);
#pragma unroll
    for (int u = 0; u < BCAST_U; ++u)
        if (pos[u] < total) __builtin_nontemporal_store(val[u], dst + pos[u]);
}

// ------------------------------------------------------------------------------------------------
// Cast fused into boxing (Sec. 6.4: sharded optimizer state with mixed precision).
// Forward, fp32 S(a) -> bf16 B: the walk of box_gather_bcast_kernel (chunked passes, one destination at
// a time, re-reads from L2) with VE elements per lane: 32 bytes in, one hardware conversion per pair
// (round to nearest even), 16 bytes out.  VE = 1 is the fallback for shapes without 8-element alignment.
// ------------------------------------------------------------------------------------------------
__device__ inline uint32_t cvt2_bf16(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <int VE>
__global__ __launch_bounds__(BOX_THREADS) void box_cast_gather_kernel(BoxParams p, uint32_t log2_pieces, uint32_t total,
                                                                       uint32_t q, uint32_t rem) {
    __shared__ const float* sp[SBP_MAX_K];
    if ((int)threadIdx.x < p.ki) sp[threadIdx.x] = static_cast<const float*>(p.src[threadIdx.x]);
    __syncthreads();
    const uint32_t k = (uint32_t)p.ko;
    const uint32_t piece = blockIdx.x & ((1u << log2_pieces) - 1);
    const uint32_t cj = blockIdx.x >> log2_pieces;
    const uint32_t chunk = cj / k, j = cj - chunk * k;
    const uint32_t idx = ((chunk << log2_pieces) + piece) * (uint32_t)BOX_THREADS + threadIdx.x;   // group of VE elements
    if (idx >= total) return;
    const uint32_t cols_v = (uint32_t)(p.cols / VE);
    const uint32_t r = idx / cols_v, c = idx - r * cols_v;
    const bool by_rows = p.axis_in == 0;
    const uint32_t x = by_rows ? r : c * VE;
    const uint32_t edge = rem * (q + 1);
    uint32_t i, begin, len;
    if (x < edge) {
        i = x / (q + 1);
        begin = i * (q + 1);
        len = q + 1;
    } else {
        i = (x - edge) / (q ? q : 1);
        begin = edge + i * q;
        i += rem;
        len = q;
    }
    const int64_t spos = by_rows ? ((int64_t)(r - begin) * p.cols + (int64_t)c * VE) : ((int64_t)r * len + (x - begin));   // elements
    const float* src = sp[i] + spos;
    if constexpr (VE == 8) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(src), b = *reinterpret_cast<const f32x4*>(src + 4);
        const u32x4 o = {cvt2_bf16(a[0], a[1]), cvt2_bf16(a[2], a[3]), cvt2_bf16(b[0], b[1]), cvt2_bf16(b[2], b[3])};
        __builtin_nontemporal_store(o, static_cast<u32x4*>(p.dst[j]) + idx);
    } else {
        static_cast<uint16_t*>(p.dst[j])[idx] = (uint16_t)(cvt2_bf16(*src, 0.0f) & 0xFFFFu);
    }
}

// Backward, bf16 P(sum) -> fp32 S(a): out_j = sum over the k partials of slice j, widened to fp32 and
// added in shard order.  Tasks as for P -> S (one per destination).
template <int VE, int KS>
__global__ __launch_bounds__(BOX_THREADS) void box_cast_reduce_kernel(BoxParams p) {
    const Task T = make_task(p, blockIdx.y);
    const int32_t ns = KS > 0 ? KS : T.ns;
    const uint32_t cols_v = (uint32_t)(T.cols / VE);
    const uint32_t total = (uint32_t)T.rows * cols_v;
    const uint32_t stride = gridDim.x * BOX_THREADS;
    float* __restrict__ dst = static_cast<float*>(p.dst[T.d0]);
    for (uint32_t idx = blockIdx.x * BOX_THREADS + threadIdx.x; idx < total; idx += stride) {
        const uint32_t r = T.rows == 1 ? 0 : idx / cols_v;
        const uint32_t c = idx - r * cols_v;
        const int64_t spos = T.src_off + (int64_t)r * T.src_ld + (int64_t)c * VE;
        const int64_t dpos = T.dst_off + (int64_t)r * T.dst_ld + (int64_t)c * VE;
        if constexpr (VE == 8) {
            float acc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
            auto add = [&](int i) {
                const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.src[i]) + spos));
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    acc[2 * d] += __uint_as_float(w[d] << 16);
                    acc[2 * d + 1] += __uint_as_float(w[d] & 0xFFFF0000u);
                }
            };
            if constexpr (KS > 0) {
#pragma unroll
                for (int i = 0; i < KS; ++i) add(i);
            } else {
                for (int i = 0; i < ns; ++i) add(i);
            }
            const f32x4 o0 = {acc[0], acc[1], acc[2], acc[3]}, o1 = {acc[4], acc[5], acc[6], acc[7]};
            __builtin_nontemporal_store(o0, reinterpret_cast<f32x4*>(dst + dpos));
            __builtin_nontemporal_store(o1, reinterpret_cast<f32x4*>(dst + dpos + 4));
        } else {
            float acc = 0.0f;
            for (int i = 0; i < ns; ++i) acc += __uint_as_float((uint32_t)static_cast<const uint16_t*>(p.src[i])[spos] << 16);
            dst[dpos] = acc;
        }
    }
}

// S(a) -> P(op), B -> P(op) (Table 2 prices them at zero on the same devices): device j keeps what it
// already holds, placed in the full-shape partial, and every other position gets the identity of
// the reduction (0 / -inf).  B: device 0 keeps its copy, the others hold the identity only.
// blockIdx.y = destination, the slow grid dimension, so the chip writes one destination at a time.
template <typename V, bool MAXOP>
__global__ __launch_bounds__(BOX_THREADS) void box_to_partial_kernel(BoxParams p, uint32_t total) {
    const int32_t j = blockIdx.y;
    const uint32_t lv = __builtin_ctz((uint32_t)p.vec_elems);
    const uint32_t cols_v = (uint32_t)(p.cols >> lv);
    int64_t rb = 0, rl = p.rows, cb = 0, cl = p.cols;
    if (p.axis_in == 0) range_of(p.rows, p.ko, j, 1, rb, rl);
    if (p.axis_in == 1) range_of(p.cols, p.ko, j, 1, cb, cl);
    if (p.axis_in < 0 && j > 0) rl = 0;   // B: only device 0 contributes
    const V* __restrict__ src = static_cast<const V*>(p.src[j]);
    V* __restrict__ dst = static_cast<V*>(p.dst[j]);
    V ident;
    if constexpr (MAXOP) ident = V(-__builtin_inff());
    else ident = V(0.0f);
    const uint32_t stride = gridDim.x * BOX_THREADS;
    for (uint32_t idx = blockIdx.x * BOX_THREADS + threadIdx.x; idx < total; idx += stride) {
        const uint32_t r = idx / cols_v, c = idx - r * cols_v;
        const int64_t x = (int64_t)c << lv;
        V v = ident;
        if ((int64_t)r >= rb && (int64_t)r < rb + rl && x >= cb && x < cb + cl)
            v = __builtin_nontemporal_load(src + ((((int64_t)r - rb) * cl + (x - cb)) >> lv));
        __builtin_nontemporal_store(v, dst + idx);
    }
}

// S(a) -> P(op) between placements of different size: output device j receives slice j of the balanced
// split of axis a over the ko OUTPUT devices (every value travels once, the table's price), so a
// position inside that slice is fetched from whichever of the ki input shards owns it.
template <typename V, bool MAXOP>
__global__ __launch_bounds__(BOX_THREADS) void box_to_partial_across_kernel(BoxParams p, uint32_t total) {
    __shared__ const V* sp[SBP_MAX_K];
    if ((int)threadIdx.x < p.ki) sp[threadIdx.x] = static_cast<const V*>(p.src[threadIdx.x]);
    __syncthreads();
    const int32_t j = blockIdx.y;
    const uint32_t lv = __builtin_ctz((uint32_t)p.vec_elems);
    const uint32_t cols_v = (uint32_t)(p.cols >> lv);
    const bool by_rows = p.axis_in == 0;
    const uint32_t n = (uint32_t)(by_rows ? p.rows : p.cols);
    const uint32_t ob = (uint32_t)split_begin(n, p.ko, j), ol = (uint32_t)split_len(n, p.ko, j);   // this device's slice
    const uint32_t q = n / (uint32_t)p.ki, rem = n % (uint32_t)p.ki, edge = rem * (q + 1);        // the input's split
    V* __restrict__ dst = static_cast<V*>(p.dst[j]);
    V ident;
    if constexpr (MAXOP) ident = V(-__builtin_inff());
    else ident = V(0.0f);
    const uint32_t stride = gridDim.x * BOX_THREADS;
    for (uint32_t idx = blockIdx.x * BOX_THREADS + threadIdx.x; idx < total; idx += stride) {
        const uint32_t r = idx / cols_v, c = idx - r * cols_v;
        const uint32_t x = by_rows ? r : c << lv;
        V v = ident;
        if (x - ob < ol) {   // unsigned: ob <= x < ob + ol
            uint32_t i, begin, len;
            if (x < edge) {
                i = x / (q + 1);
                begin = i * (q + 1);
                len = q + 1;
            } else {
                i = (x - edge) / q;   // q > 0 here: with q == 0 every index lies below edge
                begin = edge + i * q;
                i += rem;
                len = q;
            }
            const int64_t spos = by_rows ? ((int64_t)(r - begin) * p.cols + ((int64_t)c << lv)) : ((int64_t)r * len + (x - begin));
            v = __builtin_nontemporal_load(sp[i] + (spos >> lv));
        }
        __builtin_nontemporal_store(v, dst + idx);
    }
}

template <typename V>
void launch_to_partial(const BoxParams& p, bool maxop, bool across, dim3 grid, uint32_t total, hipStream_t st) {
    if (across) {
        if (maxop) hipLaunchKernelGGL((box_to_partial_across_kernel<V, true>), grid, dim3(BOX_THREADS), 0, st, p, total);
        else hipLaunchKernelGGL((box_to_partial_across_kernel<V, false>), grid, dim3(BOX_THREADS), 0, st, p, total);
    } else {
        if (maxop) hipLaunchKernelGGL((box_to_partial_kernel<V, true>), grid, dim3(BOX_THREADS), 0, st, p, total);
        else hipLaunchKernelGGL((box_to_partial_kernel<V, false>), grid, dim3(BOX_THREADS), 0, st, p, total);
    }
}

inline int64_t gcd64(int64_t a, int64_t b) {
    while (b) {
        const int64_t t = a % b;
        a = b;
        b = t;
    }
    return a < 0 ? -a : a;
}

template <typename V, int OP, int UNROLL>
void launch_reduce_k(const BoxParams& p, dim3 grid, hipStream_t st) {
    switch (p.mode == M_P2P ? 0 : p.ki) {   // P -> P walks a strided source list: run-time count
        case 2: hipLaunchKernelGGL((box_reduce_kernel<V, OP, 2, UNROLL>), grid, dim3(BOX_THREADS), 0, st, p); break;
        case 4: hipLaunchKernelGGL((box_reduce_kernel<V, OP, 4, UNROLL>), grid, dim3(BOX_THREADS), 0, st, p); break;
        case 8: hipLaunchKernelGGL((box_reduce_kernel<V, OP, 8, UNROLL>), grid, dim3(BOX_THREADS), 0, st, p); break;
        case 16: hipLaunchKernelGGL((box_reduce_kernel<V, OP, 16, UNROLL>), grid, dim3(BOX_THREADS), 0, st, p); break;
        default: hipLaunchKernelGGL((box_reduce_kernel<V, OP, 0, UNROLL>), grid, dim3(BOX_THREADS), 0, st, p); break;
    }
}

// 0 = chosen from the size (see launch_boxing); 1 / 2 / 4 / 8 = that many vectors per lane in box_reduce_kernel;
// 16 = box_reduce_diag_kernel where it exists (4, 8 or 16 sources), else 8 vectors per lane
std::atomic<int> g_box_reduce_variant{0};

template <int OP>
void launch_reduce(const BoxParams& p, dim3 grid, int unroll, hipStream_t st) {
    if (p.vec_elems == 4) {
        if (unroll == 16 && p.ki == 8) hipLaunchKernelGGL((box_reduce_diag_kernel<f32x4, OP, 8>), grid, dim3(BOX_THREADS), 0, st, p);
        else if (unroll == 16 && p.ki == 4) hipLaunchKernelGGL((box_reduce_diag_kernel<f32x4, OP, 4>), grid, dim3(BOX_THREADS), 0, st, p);
        else if (unroll == 16 && p.ki == 16) hipLaunchKernelGGL((box_reduce_diag_kernel<f32x4, OP, 16>), grid, dim3(BOX_THREADS), 0, st, p);
        else if (unroll >= 8) launch_reduce_k<f32x4, OP, 8>(p, grid, st);
        else if (unroll == 4) launch_reduce_k<f32x4, OP, 4>(p, grid, st);
        else if (unroll == 2) launch_reduce_k<f32x4, OP, 2>(p, grid, st);
        else launch_reduce_k<f32x4, OP, 1>(p, grid, st);
    } else if (p.vec_elems == 2) launch_reduce_k<f32x2, OP, 1>(p, grid, st);
    else launch_reduce_k<float, OP, 1>(p, grid, st);
}

template <typename V>
void launch_copy(const BoxParams& p, dim3 grid, int unroll, hipStream_t st) {
    if (unroll == 1) hipLaunchKernelGGL((box_copy_kernel<V, 1>), grid, dim3(BOX_THREADS), 0, st, p);
    else if (unroll == 2) hipLaunchKernelGGL((box_copy_kernel<V, 2>), grid, dim3(BOX_THREADS), 0, st, p);
    else hipLaunchKernelGGL((box_copy_kernel<V, 4>), grid, dim3(BOX_THREADS), 0, st, p);
}

}  // namespace

int32_t launch_boxing(const BoxPlan& plan, hipStream_t stream) {
    BoxParams p{};
    p.rows = plan.rows;
    p.cols = plan.cols;
    p.ki = plan.k;
    p.ko = plan.k_out;
    const int32_t ki = plan.k, ko = plan.k_out;
    p.axis_in = (plan.sbp_in == SBP_S(0) || plan.sbp_in == SBP_S(1)) ? plan.sbp_in : -1;
    p.axis_out = (plan.sbp_out == SBP_S(0) || plan.sbp_out == SBP_S(1)) ? plan.sbp_out : -1;
    const bool p_in = plan.sbp_in == SBP_P_SUM || plan.sbp_in == SBP_P_MAX;
    const bool p_out = plan.sbp_out == SBP_P_SUM || plan.sbp_out == SBP_P_MAX;
    const int32_t nb = plan.batch > 1 ? plan.batch : 1;
    // a batch: reductions only (their kernels take the conversion from blockIdx.z)
    if (nb > 1 && (!p_in || (plan.sbp_in == plan.sbp_out && ki == ko) || (int64_t)nb * (ki > ko ? ki : ko) > SBP_MAX_K)) return SBP_ERR_UNSUPPORTED;
    p.batch = nb;
    for (int i = 0; i < nb * ki; ++i) p.src[i] = plan.src[i];
    for (int i = 0; i < nb * ko; ++i) p.dst[i] = plan.dst[i];
    int32_t tasks;
    if (plan.sbp_in == plan.sbp_out && ki == ko) {
        p.mode = M_IDENT;
        p.sbp_same = plan.sbp_in;
        tasks = ki;
    } else if (p_in && p_out) {
        p.mode = M_P2P;
        tasks = ko;
    } else if (p_out) {
        // S -> P, B -> P: own values kept, identity elsewhere
        if (plan.elem_bytes != 4) return SBP_ERR_DTYPE;
        const bool across = ki != ko && p.axis_in >= 0;   // B -> P reads copy 0 only, whatever the counts
        int64_t g = 4;   // fp32 elements in 16 bytes
        g = gcd64(g, plan.cols);
        if (p.axis_in == 1) {
            for (int32_t i = 0; i < ki; ++i) {
                g = gcd64(g, split_begin(plan.cols, ki, i));
                g = gcd64(g, split_len(plan.cols, ki, i));
            }
            for (int32_t i = 0; i < ko; ++i) {
                g = gcd64(g, split_begin(plan.cols, ko, i));
                g = gcd64(g, split_len(plan.cols, ko, i));
            }
        }
        const int64_t total_v = plan.rows * plan.cols / g;
        if (total_v == 0) return SBP_OK;
        if (total_v >= ((int64_t)1 << 31) || plan.rows >= ((int64_t)1 << 31) || plan.cols >= ((int64_t)1 << 31))
            return SBP_ERR_UNSUPPORTED;
        p.vec_elems = (int32_t)g;
        int64_t bx = (total_v + BOX_THREADS - 1) / BOX_THREADS;
        const int64_t cap = (131072 + ko - 1) / ko;
        if (bx > cap) bx = cap;
        const dim3 grid((uint32_t)bx, (uint32_t)ko);
        const bool maxop = plan.sbp_out == SBP_P_MAX;
        if (g == 4) launch_to_partial<f32x4>(p, maxop, across, grid, (uint32_t)total_v, stream);
        else if (g == 2) launch_to_partial<f32x2>(p, maxop, across, grid, (uint32_t)total_v, stream);
        else launch_to_partial<float>(p, maxop, across, grid, (uint32_t)total_v, stream);
        return launch_status(__func__);
    } else if (p_in && plan.sbp_out == SBP_B) {
        p.mode = M_P2B;
        tasks = 1;
    } else if (p_in) {
        p.mode = M_P2S;
        tasks = ko;
    } else if (plan.sbp_in == SBP_B && plan.sbp_out == SBP_B) {
        // B -> B onto another device count: all-gather of a tensor "split" over one device (copy 0)
        p.mode = M_S2B;
        p.ki = 1;
        p.axis_in = 0;
        tasks = 1;
    } else if (plan.sbp_in == SBP_B) {
        p.mode = M_B2S;
        tasks = ko;
    } else if (plan.sbp_out == SBP_B) {
        p.mode = M_S2B;
        tasks = ki;
    } else {
        p.mode = M_S2S;   // also S(a) -> S(a) between different device counts
        tasks = ki * ko;
        if (p.axis_in == p.axis_out) {
            // same axis: walk the two balanced splits side by side and keep the pairs that overlap
            const int64_t n = p.axis_in == 0 ? plan.rows : plan.cols;
            int32_t i = 0, j = 0, np = 0;
            while (i < ki && j < ko) {
                const int64_t ib = split_begin(n, ki, i), ie = ib + split_len(n, ki, i);
                const int64_t jb = split_begin(n, ko, j), je = jb + split_len(n, ko, j);
                if ((ib > jb ? ib : jb) < (ie < je ? ie : je)) {
                    p.pair_i[np] = (uint8_t)i;
                    p.pair_j[np] = (uint8_t)j;
                    ++np;
                }
                if (ie <= je) ++i;
                if (je <= ie) ++j;
            }
            if (np == 0) return SBP_OK;   // an empty axis
            p.npairs = np;
            tasks = np;
        }
    }
    if (tasks > 65535) return SBP_ERR_UNSUPPORTED;

    // widest vector every task allows: all offsets, pitches and widths must be multiples of it
    int64_t g = 16 / plan.elem_bytes;  // elements in 16 bytes
    p.vec_elems = 1;                   // make_task does not depend on it
    int64_t max_units = 0;
    for (int32_t t = 0; t < tasks; ++t) {
        const Task T = make_task(p, t);
        if (T.rows * T.cols == 0) continue;
        g = gcd64(g, T.cols);
        g = gcd64(g, T.src_off);
        g = gcd64(g, T.dst_off);
        if (T.rows > 1) {
            g = gcd64(g, T.src_ld);
            g = gcd64(g, T.dst_ld);
        }
        max_units = T.rows * T.cols > max_units ? T.rows * T.cols : max_units;
    }
    if (max_units == 0) return SBP_OK;  // nothing to move
    p.vec_elems = (int32_t)g;
    max_units /= g;
    if (max_units >= (int64_t)1 << 31) return SBP_ERR_UNSUPPORTED;

    const bool reduce = p_in && p.mode != M_IDENT;
    const int vbytes = p.vec_elems * plan.elem_bytes;
    const int64_t total_v = plan.rows * plan.cols / g;
    if (p.mode == M_S2B && ko > 1 && vbytes == 16 && plan.cols % g == 0 && total_v < ((int64_t)1 << 31) &&
        plan.rows < ((int64_t)1 << 31) && plan.cols < ((int64_t)1 << 31)) {
        const int64_t per_piece = (int64_t)BOX_THREADS * BCAST_U;                 // 4 KB
        const int64_t need = (total_v + per_piece - 1) / per_piece;
        uint32_t lp = 3;                                                         // 8 .. 2048 pieces per chunk (8 MB)
        while (lp < 11 && ((int64_t)1 << lp) < need) ++lp;
        const int64_t chunks = (need + ((int64_t)1 << lp) - 1) >> lp;
        const int64_t blocks = (chunks * ko) << lp;
        if (blocks < ((int64_t)1 << 31)) {
            const int64_t n = p.axis_in == 0 ? plan.rows : plan.cols;
            hipLaunchKernelGGL(box_gather_bcast_kernel<u32x4>, dim3((uint32_t)blocks), dim3(BOX_THREADS), 0, stream, p, lp,
                               (uint32_t)total_v, (uint32_t)(n / p.ki), (uint32_t)(n % p.ki));
            return launch_status(__func__);
        }
    }
    // Vectors per lane of a reduction (16-byte vectors).  Measured on 8 sources, all-reduce, TB/s on buffers from
    // separate allocations / carved back to back from one allocation / the same with 4 KiB between them:
    //   8 x 128 MiB:  1 vector 5.76 / 4.57 / 5.59,  2: 5.18 / 5.30 / 5.55,  4: 5.61 / 5.47 / 5.58,  8: 5.43 / 5.43 / 5.40
    //   8 x 16 MiB:   1: 4.55 / 4.48 / 4.74,  4: 4.91 / 4.89 / 5.37,  8: 5.19 / 5.03 / 5.30,  sources out of phase
    //                 (box_reduce_diag_kernel): 5.36 / 5.26 / 5.43
    // One vector per lane is the fastest on large tensors unless the k buffers lie back to back (equal offsets then
    // share a memory bank, and the k stores of a lane hit it in a row); four lose 3 % there and hold up on every
    // layout, so four it is.  Medium tensors (above 8 and up to 32 MiB per source, all tasks together) take the
    // out-of-phase kernel where it exists; below that its k vectors per lane leave too few workgroups (8 partials of
    // 1 / 4 MiB: 13 / 16 us against 7.6 / 11 with four vectors per lane; 16 MiB: 45 against 49).
    int unroll = 1;
    if (reduce && vbytes == 16) {
        const int64_t all_units = max_units * tasks * nb;
        const bool medium = all_units > ((int64_t)1 << 19) && all_units <= ((int64_t)1 << 21);
        const bool diag = p.mode != M_P2P && (p.ki == 4 || p.ki == 8 || p.ki == 16);
        unroll = medium ? (diag ? 16 : 8) : 4;
        const int forced = g_box_reduce_variant.load(std::memory_order_relaxed);
        if (forced) unroll = (forced == 16 && !diag) ? 8 : forced;
    }
    const int per_lane = unroll == 16 ? p.ki : unroll;
    // Workgroups in the whole grid, at most.  A copy workgroup that moves a single 4 KB piece costs more to
    // start than to run: with 131072 of them a 2 x 512 MiB relayout ran at 3.2-4.7 TB/s, with 32768 (four
    // pieces each, grid-stride) at 5.4-6.0, and 2 x 1 GiB went from 5.5-5.7 to 5.8-5.9; 8192 is slower
    // again.  Reductions issue k loads per vector and are indifferent between 32768 and 65536.
    const int64_t cap_total = reduce ? 65536 : 32768;
    int64_t bx = (max_units + (int64_t)BOX_THREADS * per_lane - 1) / ((int64_t)BOX_THREADS * per_lane);
    const int64_t cap = (cap_total + (int64_t)tasks * nb - 1) / ((int64_t)tasks * nb);
    if (bx > cap) bx = cap;
    if (bx < 1) bx = 1;
    const dim3 grid((uint32_t)bx, (uint32_t)tasks, (uint32_t)nb);

    if (reduce) {
        if (plan.sbp_in == SBP_P_SUM) launch_reduce<BOX_SUM>(p, grid, unroll, stream);
        else launch_reduce<BOX_MAX>(p, grid, unroll, stream);
    } else {
        const int vb = vbytes;
        if (vb == 16) launch_copy<u32x4>(p, grid, unroll, stream);
        else if (vb == 8) launch_copy<u32x2>(p, grid, 4, stream);
        else if (vb == 4) launch_copy<uint32_t>(p, grid, 4, stream);
        else launch_copy<uint16_t>(p, grid, 4, stream);
    }
    return launch_status(__func__);
}

void set_box_reduce_variant(int32_t v) { g_box_reduce_variant.store(v, std::memory_order_relaxed); }

int32_t launch_boxing_cast(const BoxPlan& plan, hipStream_t stream) {
    BoxParams p{};
    p.rows = plan.rows;
    p.cols = plan.cols;
    p.ki = p.ko = plan.k;
    p.axis_in = (plan.sbp_in == SBP_S(0) || plan.sbp_in == SBP_S(1)) ? plan.sbp_in : -1;
    p.axis_out = (plan.sbp_out == SBP_S(0) || plan.sbp_out == SBP_S(1)) ? plan.sbp_out : -1;
    for (int i = 0; i < plan.k; ++i) {
        p.src[i] = plan.src[i];
        p.dst[i] = plan.dst[i];
    }
    if (plan.rows * plan.cols == 0) return SBP_OK;
    if (plan.rows >= ((int64_t)1 << 31) || plan.cols >= ((int64_t)1 << 31)) return SBP_ERR_UNSUPPORTED;
    if (p.axis_in >= 0 && plan.sbp_out == SBP_B) {
        // forward: fp32 S(a) -> bf16 B.  8 elements per lane when rows and shard boundaries allow it.
        int64_t g = gcd64(8, plan.cols);
        if (p.axis_in == 1)
            for (int32_t i = 0; i < plan.k; ++i) {
                g = gcd64(g, split_begin(plan.cols, plan.k, i));
                g = gcd64(g, split_len(plan.cols, plan.k, i));
            }
        const int ve = g == 8 ? 8 : 1;
        const int64_t total = plan.rows * plan.cols / ve;
        if (total >= ((int64_t)1 << 31)) return SBP_ERR_UNSUPPORTED;
        const int64_t need = (total + BOX_THREADS - 1) / BOX_THREADS;
        uint32_t lp = 3;
        while (lp < 11 && ((int64_t)1 << lp) < need) ++lp;
        const int64_t chunks = (need + ((int64_t)1 << lp) - 1) >> lp;
        const int64_t blocks = (chunks * plan.k) << lp;
        if (blocks >= ((int64_t)1 << 31)) return SBP_ERR_UNSUPPORTED;
        const int64_t n = p.axis_in == 0 ? plan.rows : plan.cols;
        const uint32_t q = (uint32_t)(n / plan.k), rem = (uint32_t)(n % plan.k);
        if (ve == 8)
            hipLaunchKernelGGL(box_cast_gather_kernel<8>, dim3((uint32_t)blocks), dim3(BOX_THREADS), 0, stream, p, lp, (uint32_t)total, q, rem);
        else
            hipLaunchKernelGGL(box_cast_gather_kernel<1>, dim3((uint32_t)blocks), dim3(BOX_THREADS), 0, stream, p, lp, (uint32_t)total, q, rem);
        return launch_status(__func__);
    }
    if (plan.sbp_in == SBP_P_SUM && p.axis_out >= 0) {
        // backward: bf16 P(sum) -> fp32 S(a)
        p.mode = M_P2S;
        p.vec_elems = 1;
        int64_t g = 8, max_units = 0;
        for (int32_t t = 0; t < plan.k; ++t) {
            const Task T = make_task(p, t);
            if (T.rows * T.cols == 0) continue;
            g = gcd64(g, T.cols);
            g = gcd64(g, T.src_off);
            g = gcd64(g, T.dst_off);
            if (T.rows > 1) {
                g = gcd64(g, T.src_ld);
                g = gcd64(g, T.dst_ld);
            }
            max_units = T.rows * T.cols > max_units ? T.rows * T.cols : max_units;
        }
        if (max_units == 0) return SBP_OK;
        const int ve = g == 8 ? 8 : 1;
        max_units /= ve;
        if (max_units >= ((int64_t)1 << 31)) return SBP_ERR_UNSUPPORTED;
        int64_t bx = (max_units + BOX_THREADS - 1) / BOX_THREADS;
        const int64_t cap = (65536 + plan.k - 1) / plan.k;
        if (bx > cap) bx = cap;
        const dim3 grid((uint32_t)bx, (uint32_t)plan.k);
        if (ve == 8 && plan.k == 8) hipLaunchKernelGGL((box_cast_reduce_kernel<8, 8>), grid, dim3(BOX_THREADS), 0, stream, p);
        else if (ve == 8) hipLaunchKernelGGL((box_cast_reduce_kernel<8, 0>), grid, dim3(BOX_THREADS), 0, stream, p);
        else hipLaunchKernelGGL((box_cast_reduce_kernel<1, 0>), grid, dim3(BOX_THREADS), 0, stream, p);
        return launch_status(__func__);
    }
    return SBP_ERR_UNSUPPORTED;
}

}  // namespace sbp
