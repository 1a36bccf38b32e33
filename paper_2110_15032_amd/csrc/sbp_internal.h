// Internal declarations shared by the translation units of libsbp_mi355x.so.
// Nothing here is part of the C ABI (that is include/sbp.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sbp.h"

namespace sbp {

// Balanced split (paper Sec. 3.1, "in a balanced manner"): floor(n/k) indices per shard,
// the first n mod k shards one more.  begin(k) == n.
__host__ __device__ inline int64_t split_begin(int64_t n, int32_t k, int32_t i) {
    const int64_t q = n / k, r = n % k;
    return (int64_t)i * q + (i < r ? i : r);
}
__host__ __device__ inline int64_t split_len(int64_t n, int32_t k, int32_t i) {
    return n / k + (i < n % k ? 1 : 0);
}

// Status of the launch just made; a failure is reported on stderr with HIP's own text (it means a
// launch configuration the device refused, never a data-dependent condition).
inline int32_t launch_status(const char* where) {
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return SBP_OK;
    fprintf(stderr, "libsbp_mi355x: kernel launch in %s failed: %s\n", where, hipGetErrorString(e));
    return SBP_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------------------
// Boxing: every conversion is a set of rectangle tasks.  Task t reads a rows x cols rectangle
// from n_src source shards (all at the same offset / leading dimension), combines them
// (copy when n_src == 1, sum or max in shard order otherwise) and writes the result to n_dst
// destination shards (all at the same offset / leading dimension).
// ---------------------------------------------------------------------------------------------
enum BoxOp : int32_t { BOX_COPY = 0, BOX_SUM = 1, BOX_MAX = 2 };

struct BoxPlan {
    const void* src[SBP_MAX_K];
    void* dst[SBP_MAX_K];
    int64_t rows, cols;       // global shape, in elements
    int32_t k;                // devices holding the input
    int32_t k_out;            // devices holding the output (= k on one device set; launch_boxing_cast ignores it)
    int32_t sbp_in, sbp_out;  // sbp_t values
    int32_t elem_bytes;       // 2 or 4
    // batch > 1: that many independent conversions of equal shape and signature in one launch (the groups of a
    // device grid): conversion b reads src[b * k + i] and writes dst[b * k_out + j]; batch * max(k, k_out) <=
    // SBP_MAX_K.  Only reductions (P input) take it; launch_boxing returns SBP_ERR_UNSUPPORTED, before anything is
    // enqueued, for any other conversion, and the caller then launches the conversions one by one.
    int32_t batch;
};

int32_t launch_boxing(const BoxPlan& plan, hipStream_t stream);
void set_box_reduce_variant(int32_t v);
// fp32 S(a) -> bf16 B (cast + all-gather) and bf16 P(sum) -> fp32 S(a) (cast + reduce-scatter); elem_bytes unused
int32_t launch_boxing_cast(const BoxPlan& plan, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// Grouped GEMM: shard g computes C_g[m, n] = sum_kk A_g[m, kk] * B_g[kk, n].
// a_kc: A is stored [m][kk] (kk contiguous, lda = row pitch) else [kk][m].
// b_kc: B is stored [n][kk] (kk contiguous) else [kk][n].      C is always [m][n], pitch ldc.
// ---------------------------------------------------------------------------------------------
struct GemmShard {
    const void* a;
    const void* b;
    void* c;
    float* rowmax;   // EPI_ROWMAX only: [m] fp32, max over this shard's columns of the stored results
    int32_t m, n, kk;
    int32_t lda, ldb, ldc;
};
// internal epilogue code next to the public SBP_EPI_*: store, and fold every stored row into rowmax
constexpr int32_t EPI_ROWMAX = 2;
struct GemmPlan {
    GemmShard s[SBP_MAX_K];
    int32_t groups;
    int32_t in_dtype;   // SBP_F32 | SBP_BF16
    int32_t f32_operand;  // 0: both operands have in_dtype; 1 / 2: A / B is an fp32 P(sum) partial next to a bf16 operand
    int32_t out_dtype;  // SBP_F32 | SBP_BF16
    int32_t a_kc, b_kc;
    int32_t epilogue;   // SBP_EPI_*
};

int32_t launch_gemm(const GemmPlan& plan, int32_t variant, hipStream_t stream);
void set_tile_order(int32_t order);
// The ping-pong persistent kernel (gemm_pingpong_kernel.hip).  The caller has checked: bf16 operands, every
// local reduction length a multiple of 128, operand row pitches of 16 bytes.  order: tile walk (see map_tile).
int32_t launch_gemm_pingpong(const GemmPlan& plan, int max_m, int max_n, int order, hipStream_t stream);
// Compute units of the current device, asked of the runtime once per device and kept.
int compute_units();
// Diagnostic matrix-pipe loop (probe_kernels.hip); scratch: 1 MiB of device memory.
int32_t launch_probe_mfma(int32_t mode, int32_t iters, int32_t zero, void* scratch, hipStream_t stream);
// The same with the staging memory in a static device array of the library (modes 0-6); out: 1 MiB.
int32_t launch_probe_mfma_static(int32_t mode, int32_t iters, int32_t zero, void* out, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// Row statistics of the model-parallel softmax.
// ---------------------------------------------------------------------------------------------
struct RowStatPlan {
    const void* logits[SBP_MAX_K];
    const float* gmax[SBP_MAX_K];   // null for the max pass
    float* out[SBP_MAX_K];
    int32_t cols[SBP_MAX_K];        // local column count of every shard
    int32_t ld[SBP_MAX_K];          // row pitch of every shard, elements
    int64_t rows;
    int32_t k;
    int32_t dtype;
};
// Sparse cross entropy on S(1) logits.  Arrays sized for 32 shards keep the argument block small.
constexpr int XENT_MAX_K = 32;
struct XentPlan {
    const void* logits[XENT_MAX_K];
    const int32_t* labels[XENT_MAX_K];
    const float* gmax[XENT_MAX_K];
    const float* denom[XENT_MAX_K];
    const float* grad[XENT_MAX_K];   // backward only
    void* out[XENT_MAX_K];           // loss partials (f32) or dlogits (dtype)
    int32_t cols[XENT_MAX_K];        // local column count
    int32_t ld[XENT_MAX_K];          // row pitch of the logits, elements
    int32_t ld_out[XENT_MAX_K];      // row pitch of dlogits (backward only)
    int32_t begin[XENT_MAX_K];       // first global column of the shard
    int64_t rows;
    int32_t total_cols;
    int32_t k;
    int32_t dtype;
};
int32_t launch_xent_loss(const XentPlan& plan, hipStream_t stream);
int32_t launch_xent_grad(const XentPlan& plan, hipStream_t stream);

int32_t launch_row_stat(const RowStatPlan& plan, bool sumexp, hipStream_t stream);

}  // namespace sbp
