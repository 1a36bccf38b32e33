/*
 * sbp.h -- C ABI of the MI355X (gfx950) SBP matmul + boxing library.
 *
 * Vocabulary (OneFlow paper, arXiv 2110.15032, Sec. 3.1): a *global* (logical)
 * tensor placed on k devices is represented by k *local* tensors, related by an
 * SBP signature:
 *     split(a)       S(a): locals are a balanced split of the global along axis a
 *     broadcast      B   : every local is an exact copy of the global
 *     partial-value  P(op): locals have the global shape, global = elementwise
 *                           op (sum | max) over all locals
 * Here the k devices are k shard buffers in ONE GPU's memory.
 *
 * Conventions for every function:
 *   - extern "C"; returns an int32 status: SBP_OK (0) or a negative SBP_ERR_*.
 *     On any error nothing has been enqueued.  Nothing throws.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work
 *     is enqueued on it; no call synchronises, none allocates device memory.
 *   - sbp_tensor_t.shard is a HOST array of k DEVICE pointers.  The caller owns
 *     the array and every buffer; the library reads the array during the call
 *     only.  Every device pointer must be 16-byte aligned.
 *   - Local tensors are dense and row-major.  Shard i's local shape follows
 *     from (rows, cols, sbp, k, i): S(0) -> rows split, S(1) -> cols split,
 *     B / P -> full shape.  The split is the balanced one: floor(n/k) indices
 *     each, the first (n mod k) shards one more (the paper only says
 *     "balanced"; this is the reading taken).
 *   - trans = 1: shard i stores the TRANSPOSE of logical local tensor i
 *     (row-major [local_cols, local_rows]).  rows / cols / sbp always describe
 *     the logical tensor.
 *   - Output buffers must not overlap input buffers (SBP_ERR_ALIAS).  A B input
 *     may name the same buffer k times (one physical copy standing for k).
 *   - Boxing is never implicit: sbp_matmul writes Y under exactly the signature
 *     Table 1 gives; converting it is a separate sbp_boxing call, as in the
 *     paper where the compiler or to_global() inserts the boxing op (Sec. 3.2,
 *     Sec. 3.4).
 */
#ifndef SBP_MI355X_H
#define SBP_MI355X_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- SBP signatures -------------------------------------------------------*/
typedef int32_t sbp_t;
#define SBP_S(axis) ((sbp_t)(axis)) /* axis = 0 | 1 */
#define SBP_B       ((sbp_t)-1)
#define SBP_P_SUM   ((sbp_t)-2)
#define SBP_P_MAX   ((sbp_t)-3)
#define SBP_AUTO    ((sbp_t)-100)   /* sbp_matmul only: "whatever Table 1 says" */

/* ---- element types --------------------------------------------------------*/
enum { SBP_F32 = 0, SBP_BF16 = 1, SBP_I32 = 2 /* class labels of sbp_xent_* only */ };

/* ---- status codes ---------------------------------------------------------*/
enum {
    SBP_OK = 0,
    SBP_ERR_NULL = -1,        /* null descriptor, shard array or shard pointer          */
    SBP_ERR_K = -2,           /* k < 1 or k > SBP_MAX_K                                  */
    SBP_ERR_SHAPE = -3,       /* negative extent, or operand shapes do not compose       */
    SBP_ERR_DTYPE = -4,       /* unknown dtype, or dtype not allowed in that position    */
    SBP_ERR_AXIS = -5,        /* not a signature (split axis other than 0 / 1, ...)      */
    SBP_ERR_SIGNATURE = -6,   /* (sbp_x, sbp_w) not in Table 1, or sbp_y != the deduced  */
    SBP_ERR_ALIAS = -7,       /* an output buffer overlaps an input or another output    */
    SBP_ERR_ALIGN = -8,       /* a device pointer is not 16-byte aligned                 */
    SBP_ERR_UNSUPPORTED = -9, /* a valid request this build has no kernel for            */
    SBP_ERR_LAUNCH = -10      /* the HIP runtime refused the launch                      */
};
#define SBP_MAX_K 64

/* ---- a global tensor and its k local tensors ------------------------------*/
typedef struct sbp_tensor {
    void* const* shard; /* host array [k] of device pointers                          */
    int64_t rows, cols; /* GLOBAL shape; vectors are [n, 1]                           */
    int32_t dtype;      /* SBP_F32 | SBP_BF16 (SBP_I32 for label vectors)             */
    int32_t trans;      /* 0: shards hold the local tensor; 1: its transpose          */
    int64_t ld;         /* row pitch of every stored local buffer in elements, 0 = dense
                           (the stored row length).  Must be at least the longest stored row of
                           any shard (SBP_ERR_SHAPE otherwise); the bytes between a row's end and
                           the next row are never read or written.  A pitch that is a multiple of
                           128 bytes keeps every row on cache-line boundaries (the classifier's
                           125000-column logits shards: pitch 125056).  Accepted by sbp_matmul,
                           sbp_matmul_ex, sbp_matmul_rowmax, sbp_matmul_2d, sbp_row_max,
                           sbp_row_sumexp, sbp_xent_loss and sbp_xent_grad; the boxing entry
                           points take dense tensors only (SBP_ERR_UNSUPPORTED).                */
} sbp_tensor_t;

/* ---- epilogues of sbp_matmul_ex -------------------------------------------*/
enum {
    SBP_EPI_NONE = 0,
    SBP_EPI_GELU = 1    /* y <- gelu(acc), exact erf form, evaluated in fp32 on the accumulator
                           before the single rounding to y's dtype.  Elementwise, so only allowed
                           when Y is S or B (an elementwise nonlinearity of a P(sum) partial is
                           not the nonlinearity of the global value).                           */
};

/* Table 1 of the paper (Sec. 3.1): the signature of Y = XW from those of X and W.
 * Valid pairs: (S0,B)->S0, (B,S1)->S1, (S1,S0)->P(sum), (P(sum),B)->P(sum),
 * (B,P(sum))->P(sum), (B,B)->B.  Host only.  SBP_ERR_SIGNATURE for any other pair. */
int32_t sbp_infer_matmul(sbp_t sbp_x, sbp_t sbp_w, sbp_t* sbp_y);

/* Local shape of shard i (Sec. 3.1, balanced split).  Host only. */
int32_t sbp_local_shape(int64_t rows, int64_t cols, sbp_t sbp, int32_t k, int32_t i,
                        int64_t* local_rows, int64_t* local_cols);

/* Y = XW under SBP (Sec. 3.1, Table 1): every device i multiplies the local
 * tensors it holds, Y_i = X_i W_i, in ONE grouped launch over the k shards.
 *   x [M,K], w [K,N], y [M,N] global shapes; x and w share a dtype (but see P(sum)
 *   operands below).
 *   sbp_y must be the Table-1 result or SBP_AUTO.
 *   dtype of y: P(sum) results are always SBP_F32 (un-reduced partials keep the
 *   accumulator's precision); S / B results have the inputs' dtype.  bf16
 *   inputs accumulate in fp32 and round once, to nearest even.
 *   A P(sum) input operand (rows 4, 5 of Table 1) must be SBP_F32; the other
 *   operand (B) may be SBP_F32 or SBP_BF16.  Next to a bf16 operand the fp32
 *   partial is not rounded: it enters the matrix units as an exact sum of three
 *   bf16 terms.  The same holds for row 6 when one B operand is SBP_F32 (a
 *   partial that was boxed to B) and the other SBP_BF16; the result is then
 *   SBP_F32.  Any other mix of dtypes is SBP_ERR_DTYPE.
 *   k-way results are written to y->shard[i]; x, w are read only. */
int32_t sbp_matmul(const sbp_tensor_t* x, sbp_t sbp_x, const sbp_tensor_t* w, sbp_t sbp_w,
                   const sbp_tensor_t* y, sbp_t sbp_y, int32_t k, void* stream);

/* sbp_matmul with an elementwise epilogue fused before the store (SBP_EPI_*). */
int32_t sbp_matmul_ex(const sbp_tensor_t* x, sbp_t sbp_x, const sbp_tensor_t* w, sbp_t sbp_w,
                      const sbp_tensor_t* y, sbp_t sbp_y, int32_t k, void* stream,
                      int32_t epilogue);

/* sbp_matmul for a column-split result (Table 1 row 2, sbp_y = S(1) or SBP_AUTO) that also
 * delivers the first statistic of the model-parallel softmax (Sec. 6.3.1): rowmax [M,1] f32,
 * P(max), rowmax_i[r] = max over the columns device i holds of y as stored (for bf16 results: of
 * the rounded values), exactly what sbp_row_max(y) gives, without the second pass over y where
 * the GEMM kernel can fold it into its stores.  rowmax shards must not overlap x, w or y. */
int32_t sbp_matmul_rowmax(const sbp_tensor_t* x, sbp_t sbp_x, const sbp_tensor_t* w, sbp_t sbp_w,
                          const sbp_tensor_t* y, sbp_t sbp_y, const sbp_tensor_t* rowmax, int32_t k,
                          void* stream);

/* Boxing (Sec. 3.2, Table 2, same device set): rewrite the k local tensors of one
 * global tensor from sbp_in to sbp_out; the global tensor is unchanged.
 *   P(sum)/P(max) -> B      all-reduce:      out_j = op_i in_i            for every j
 *   P(sum)/P(max) -> S(a)   reduce-scatter:  out_j = op_i in_i[slice_j]
 *   S(a) -> B               all-gather:      out_j = concat_i in_i        for every j
 *   S(a) -> S(b), a != b    all2all:         out_j = concat_i in_i[slice_j along b]
 *   B -> S(a)               local slice:     out_j = in_j[slice_j]  (its OWN copy)
 *   S(a)->S(a), B->B, P->P  identity copies
 *   S(a) -> P(op), B -> P(op)     zero-cost forms: every device keeps the values it
 *                           already holds, placed in a full-shape partial, and fills
 *                           the rest with the identity of op (0 for sum, -inf for max);
 *                           from B, device 0 keeps its copy and the others hold only
 *                           the identity.
 * in->rows/cols/dtype must equal out's; P tensors must be SBP_F32; reductions are
 * done in fp32 in shard order i = 0 .. k-1, so every B copy is bit-identical and
 * runs are bit-reproducible.  P(max), here and in the row maxima below: a NaN next
 * to a number is ignored, and the maximum of +0 and -0 may carry either sign.  When
 * every operand is NaN, sbp_boxing gives NaN; sbp_row_max and sbp_matmul_rowmax start
 * from the identity and give -inf.  S/B -> S/B moves raw words and never interprets
 * them (NaN patterns survive).  trans must be 0 on both sides. */
int32_t sbp_boxing(const sbp_tensor_t* in, sbp_t sbp_in, const sbp_tensor_t* out, sbp_t sbp_out,
                   int32_t k, void* stream);

/* Boxing between DISJOINT placements (Sec. 3.2, Table 2, column "disjoint"): the input's local
 * tensors live on k_in logical devices, the output's on k_out other ones; the global tensor is
 * unchanged.  in->shard holds k_in pointers, out->shard k_out; the balanced split of an S
 * signature uses its own side's device count.  Everything sbp_boxing states about dtypes,
 * fp32 reductions in input order, raw-word moves, trans and aliasing holds here too.
 *   S(a)/B/P -> S(b), B     out = scatter(assemble(in)) over k_out devices; from B every value
 *                           is read from ONE copy (slice j from copy j mod k_in; B -> B from copy 0)
 *   S(a) -> P(op)           out_j = slice j of the balanced split of axis a over the k_out devices,
 *                           identity of op elsewhere            (every value travels once)
 *   B -> P(op)              out_0 = a copy, the others hold the identity
 *   P(op) -> P(op)          partial i goes whole to out_(i mod k_out); a device that receives
 *                           several combines them in input order, one that receives none holds
 *                           the identity                        (each partial travels once)
 * With k_in == k_out every result equals sbp_boxing's.  The paper prices these moves but does not
 * say where a P output's values land; the three P rows above are the placements that move exactly
 * the priced amount. */
int32_t sbp_boxing_across(const sbp_tensor_t* in, sbp_t sbp_in, int32_t k_in, const sbp_tensor_t* out,
                          sbp_t sbp_out, int32_t k_out, void* stream);

/* Precision cast fused into boxing (Sec. 6.4, sharded optimizer state with mixed
 * precision: the cast op's input is S(0) and its output B).
 *   forward:   in SBP_F32  S(a)    -> out SBP_BF16 B     out_j = bf16(concat_i in_i), every j;
 *              one rounding to nearest even (cast + all-gather in one pass)
 *   backward:  in SBP_BF16 P(sum)  -> out SBP_F32  S(a)  out_j = sum_i f32(in_i)[slice_j];
 *              widened exactly, added in fp32 in shard order (cast + reduce-scatter)
 * Same shape, ownership and alias rules as sbp_boxing.  Any other pair of signatures
 * is SBP_ERR_SIGNATURE, any other pair of dtypes SBP_ERR_DTYPE. */
int32_t sbp_boxing_cast(const sbp_tensor_t* in, sbp_t sbp_in, const sbp_tensor_t* out, sbp_t sbp_out,
                        int32_t k, void* stream);

/* Two-dimensional SBP (Sec. 3.3, Table 3).  The logical devices form a k0 x k1 grid (k0 groups
 * of k1 devices, k0 * k1 <= SBP_MAX_K); a signature is a pair s[2] = (outer, inner): the outer
 * entry places the tensor on the k0 groups, the inner entry places each group's tensor on its
 * k1 devices (balanced splits, nested).  Device (a, b) is shard[a * k1 + b].  trans must be 0.
 *
 * sbp_infer_matmul_2d: Table 1 applied to each grid axis on its own; Table 3's two rows,
 *   ((S0,B),(B,S1)) -> (S0,S1) and ((S0,S1),(B,S0)) -> (S0,P(sum)), are two instances.
 * sbp_matmul_2d: every device multiplies the two local tensors it holds (one grouped launch).
 *   sbp_y may be NULL or hold SBP_AUTO entries; otherwise it must equal the deduced pair.
 *   dtype rules as for sbp_matmul (a tensor with P(sum) in either position is SBP_F32).
 * sbp_boxing_2d: boxing along ONE grid axis; the other entry of the signature must stay.
 *   Inner entry changes: every group re-arranges its own tensor.  Outer entry changes: the
 *   devices with equal inner index b are boxed among themselves (with inner entry B they hold the
 *   whole tensor under the outer signature, with inner entry P(op) one op-term of it, with inner
 *   entry S(d) slice b of it provided neither outer entry is S(d)).  SBP_ERR_UNSUPPORTED: an outer
 *   conversion along the inner split's own axis; reducing an outer P(op) while the inner entry is a
 *   partial of the OTHER operation (the signature means outer-op over groups of inner-op over
 *   devices, and sum and max do not commute); changing both entries in one call.  Every part is
 *   validated before any is enqueued. */
int32_t sbp_infer_matmul_2d(const sbp_t* sbp_x, const sbp_t* sbp_w, sbp_t* sbp_y);
int32_t sbp_local_shape_2d(int64_t rows, int64_t cols, const sbp_t* sbp, int32_t k0, int32_t k1,
                           int32_t a, int32_t b, int64_t* local_rows, int64_t* local_cols);
int32_t sbp_matmul_2d(const sbp_tensor_t* x, const sbp_t* sbp_x, const sbp_tensor_t* w, const sbp_t* sbp_w,
                      const sbp_tensor_t* y, const sbp_t* sbp_y, int32_t k0, int32_t k1, void* stream);
int32_t sbp_boxing_2d(const sbp_tensor_t* in, const sbp_t* sbp_in, const sbp_tensor_t* out, const sbp_t* sbp_out,
                      int32_t k0, int32_t k1, void* stream);

/* Local reductions of the model-parallel softmax (Sec. 6.3.1): logits [R, C] are
 * S(1); each device reduces the columns it holds.
 *   sbp_row_max:    m_i[r] = max_c L_i[r, c]              -> out [R,1] f32, P(max)
 *   sbp_row_sumexp: s_i[r] = sum_c exp(L_i[r, c] - m[r])  -> out [R,1] f32, P(sum)
 * gmax is the B tensor [R,1] f32 obtained by boxing the P(max) to B.  Statistics
 * are taken over the logits as stored (bf16 or f32), in fp32.  A device that
 * holds no column writes the identity (-inf, 0).  sbp_l other than S(1) does not
 * yield partial vectors and is rejected with SBP_ERR_UNSUPPORTED. */
int32_t sbp_row_max(const sbp_tensor_t* logits, sbp_t sbp_l, const sbp_tensor_t* out,
                    int32_t k, void* stream);
int32_t sbp_row_sumexp(const sbp_tensor_t* logits, sbp_t sbp_l, const sbp_tensor_t* gmax,
                       const sbp_tensor_t* out, int32_t k, void* stream);

/* Sparse cross entropy on the same model-parallel logits (Sec. 6.3.1: MatMul, softmax and sparse
 * cross entropy with the weight S(1)).  logits [R,C] S(1), bf16 or f32.  labels [R,1] SBP_I32, B:
 * the class of every row; a value outside [0, C) marks a row that is ignored.  gmax, denom [R,1]
 * f32, B: the global row max and softmax denominator (sbp_row_max / sbp_row_sumexp, each boxed to
 * B).  Vectors are passed as k device pointers like every B tensor (copies may share one buffer).
 *   sbp_xent_loss: loss [R,1] f32 P(sum).  The device that holds column y[r] writes
 *                  log denom[r] + gmax[r] - L[r, y[r]], every other device (and every ignored
 *                  row) 0; boxing P(sum) -> B gives -log softmax(L[r,:])[y[r]].
 *   sbp_xent_grad: dlogits [R,C] S(1), dtype of logits:
 *                  (exp(L[r,c] - gmax[r]) / denom[r] - [c == y[r]]) * grad[r], grad [R,1] f32 B the
 *                  upstream gradient of every row's loss; ignored rows get 0.  Elementwise, no
 *                  communication.  One rounding to nearest even for bf16.
 * At most 32 devices (SBP_ERR_UNSUPPORTED beyond); sbp_l other than S(1) as for sbp_row_max. */
int32_t sbp_xent_loss(const sbp_tensor_t* logits, sbp_t sbp_l, const sbp_tensor_t* labels, const sbp_tensor_t* gmax,
                      const sbp_tensor_t* denom, const sbp_tensor_t* loss, int32_t k, void* stream);
int32_t sbp_xent_grad(const sbp_tensor_t* logits, sbp_t sbp_l, const sbp_tensor_t* labels, const sbp_tensor_t* gmax,
                      const sbp_tensor_t* denom, const sbp_tensor_t* grad, const sbp_tensor_t* dlogits, int32_t k,
                      void* stream);

/* Tuning knobs; they never change what is computed beyond fp32 summation order
 * inside a GEMM tile.  Unknown knob or value: SBP_ERR_UNSUPPORTED. */
enum {
    SBP_KNOB_GEMM_VARIANT = 0,  /* 0 = default choice by shape; >0 forces a kernel: 1 generic, 3 = 256x256
                                   tile with two 64-deep stages, 4 = 128x128 tile, 6 = 256x256 with four
                                   32-deep stages, 7 = 6 on the 16x16x32 matrix instruction,
                                   12 = 6 as one persistent workgroup per compute unit
                                   (needs every local reduction length to be a multiple of 128), 16 =
                                   12 on the 16x16x32 matrix instruction, 21 = 16 with the two waves of
                                   every SIMD taking turns at the matrix pipe (ping-pong); a forced
                                   kernel that cannot take the shapes gives SBP_ERR_UNSUPPORTED        */
    SBP_KNOB_TILE_ORDER = 1,    /* order in which workgroups walk output tiles: low byte = tile-rows per
                                   band (0, the default: chosen from the shape), bit 8 set = no per-XCD
                                   re-linearisation                                                     */
    SBP_KNOB_BOX_REDUCE = 2     /* 16-byte vectors per lane in the reductions of sbp_boxing: 0 = chosen
                                   from the size, 1 / 2 / 4 / 8, or 16 = the kernel that reads the k
                                   sources out of phase (4, 8 or 16 sources; 8 per lane otherwise).  The
                                   sums are the same bit for bit under every value.                     */
};
/* The knobs are process-wide settings read at every call (atomically); a caller that changes one while
 * another thread is inside the library gets either value for that call.  They are meant for measurement. */
int32_t sbp_set_knob(int32_t knob, int32_t value);

/* Diagnostic, not part of the method: a loop of matrix instructions alone, to measure what the chip's matrix
 * pipes sustain and what operand fragment reads between the instructions cost (context for the rates that
 * sbp_matmul reaches; bench.py --workload mfma_probe reports it).  One workgroup of 8 waves per compute unit;
 * every wave runs `iters` rounds of 32 v_mfma_f32_16x16x32_bf16 (2 * 16 * 16 * 32 flop each per wave).
 *   mode 0: matrix instructions only; 1: with 16 LDS fragment reads per round interleaved in both waves of a
 *   SIMD and a barrier per round (lockstep schedule); 2: the two waves of a SIMD alternating between their
 *   reads and their matrix instructions (ping-pong schedule); 3: as 0 with 16 v_mfma_f32_32x32x16_bf16 per
 *   round (same flop); 4, 5: as 2 with 12 and with 8 fragment reads per round; 6: as 4 plus an operand stream
 *   of 32 KB per compute unit and round from (L2-resident) global memory straight into LDS; 7: as 6 with 8 of
 *   those 32 KB from a 1 GiB region that misses every cache; 8: as 7 plus 4 KB of streaming stores per compute
 *   unit and round.
 *   zero_operands != 0: all-zero fragments instead of pseudo-random ones (no operand toggling).
 *   scratch: 1 MiB of device memory (mode 6: 16 MiB; modes 7, 8: 16 MiB + 1.5 GiB), 16-byte aligned, caller-owned; after the call has completed its first
 *   8 uint64 words hold the shader cycles each wave of workgroup 0 spent in the loop.
 * Total flop of a call: compute units * 8 * iters * 32 * 16384. */
int32_t sbp_probe_mfma(int32_t mode, int32_t iters, int32_t zero_operands, void* scratch, void* stream);

/* sbp_probe_mfma for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels, modes 0 to 6, with the staging memory of mode 6 in a
 * static device array inside the library (15 MiB per device the library runs on, held until the process ends)
 * instead of a caller workspace.  The call allocates nothing, neither itself nor through the runtime calls it
 * makes (on its first call on a device it asks the runtime for the array's address and keeps it).
 *   out: 1 MiB of device memory, 16-byte aligned, caller-owned: 8 uint64 words (shader cycles of the waves of
 *        workgroup 0), then from byte 64 one float per thread of the grid (compute units * 512): the sum of the
 *        thread's accumulators, a pure function of (mode, iters, zero_operands) and equal, bit for bit, to what
 *        sbp_probe_mfma leaves at the same place of its scratch.
 * SBP_ERR_UNSUPPORTED: modes 7 and 8 (they walk 1.5 GiB), iters outside 1 .. 2^24, or a device with more than
 * 480 compute units (32 KB of the array each); nothing is launched then.
 * All calls on one device share that device's array and keep no state in it between calls (mode 6 fills the part
 * it reads before reading it); calls that overlap in time on one device race on it. */
int32_t sbp_probe_mfma_static(int32_t mode, int32_t iters, int32_t zero_operands, void* out, void* stream);

/* Static, NUL-terminated description of a status code. */
const char* sbp_strerror(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* SBP_MI355X_H */
