// Host side of the C ABI: argument validation, Table-1 deduction, shard geometry and dispatch.
// Every check runs before anything is enqueued, so a failed call has no effect on the stream.
#include <algorithm>
#include <atomic>
#include <vector>

#include "sbp_internal.h"

namespace {

using namespace sbp;

std::atomic<int32_t> g_gemm_variant{0};

bool is_sbp(sbp_t s) { return s == SBP_S(0) || s == SBP_S(1) || s == SBP_B || s == SBP_P_SUM || s == SBP_P_MAX; }
bool is_partial(sbp_t s) { return s == SBP_P_SUM || s == SBP_P_MAX; }
int elem_bytes(int32_t dtype) { return dtype == SBP_BF16 ? 2 : 4; }

struct Local {
    int64_t rows, cols;
};
Local local_of(int64_t rows, int64_t cols, sbp_t s, int32_t k, int32_t i) {
    if (s == SBP_S(0)) return {split_len(rows, k, i), cols};
    if (s == SBP_S(1)) return {rows, split_len(cols, k, i)};
    return {rows, cols};
}

// row pitch of a stored local buffer in elements: the descriptor's, or the stored row length
int64_t pitch_of(const sbp_tensor_t* t, const Local& l) { return t->ld ? t->ld : (t->trans ? l.rows : l.cols); }

// with_ld: the entry point takes a row pitch (sbp_tensor_t::ld); the others want dense tensors
int32_t check_tensor(const sbp_tensor_t* t, sbp_t s, int32_t k, bool with_ld = false) {
    if (!t || !t->shard) return SBP_ERR_NULL;
    if (t->rows < 0 || t->cols < 0 || t->ld < 0) return SBP_ERR_SHAPE;
    if (t->dtype != SBP_F32 && t->dtype != SBP_BF16) return SBP_ERR_DTYPE;
    if (t->trans != 0 && t->trans != 1) return SBP_ERR_SHAPE;
    if (!is_sbp(s)) return SBP_ERR_AXIS;
    if (t->ld && !with_ld) return SBP_ERR_UNSUPPORTED;
    if (t->ld > INT32_MAX) return SBP_ERR_UNSUPPORTED;
    for (int32_t i = 0; i < k; ++i) {
        const Local l = local_of(t->rows, t->cols, s, k, i);
        if (l.rows * l.cols == 0) continue;  // an empty local tensor needs no storage
        if (t->ld && (t->trans ? l.rows : l.cols) > t->ld) return SBP_ERR_SHAPE;
        if (!t->shard[i]) return SBP_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(t->shard[i]) & 15u) return SBP_ERR_ALIGN;
    }
    return SBP_OK;
}

struct Span {
    uintptr_t lo, hi;
};
void spans_of(const sbp_tensor_t* t, sbp_t s, int32_t k, std::vector<Span>& v) {
    for (int32_t i = 0; i < k; ++i) {
        const Local l = local_of(t->rows, t->cols, s, k, i);
        if (l.rows * l.cols == 0) continue;
        // stored as nrow rows of ncol elements, pitch_of() apart: the span ends with the last row's last element
        const int64_t nrow = t->trans ? l.cols : l.rows, ncol = t->trans ? l.rows : l.cols;
        const uintptr_t bytes = (uintptr_t)((nrow - 1) * pitch_of(t, l) + ncol) * elem_bytes(t->dtype);
        const uintptr_t lo = reinterpret_cast<uintptr_t>(t->shard[i]);
        v.push_back({lo, lo + bytes});
    }
}
bool overlap(const Span& a, const Span& b) { return a.lo < b.hi && b.lo < a.hi; }

// Two-dimensional signatures (Sec. 3.3): s[0] places the tensor on the k0 groups, s[1] each group's
// tensor on its k1 devices; device (a, b) is shard a * k1 + b.
Local local_of2(int64_t rows, int64_t cols, const sbp_t* s, int32_t k0, int32_t k1, int32_t a, int32_t b) {
    const Local n = local_of(rows, cols, s[0], k0, a);
    return local_of(n.rows, n.cols, s[1], k1, b);
}
int32_t check_grid(int32_t k0, int32_t k1) {
    if (k0 < 1 || k1 < 1 || (int64_t)k0 * k1 > SBP_MAX_K) return SBP_ERR_K;
    return SBP_OK;
}
int32_t check_tensor2(const sbp_tensor_t* t, const sbp_t* s, int32_t k0, int32_t k1, bool with_ld = false) {
    if (!t || !t->shard || !s) return SBP_ERR_NULL;
    if (t->rows < 0 || t->cols < 0 || t->ld < 0) return SBP_ERR_SHAPE;
    if (t->dtype != SBP_F32 && t->dtype != SBP_BF16) return SBP_ERR_DTYPE;
    if (t->trans != 0 || (t->ld != 0 && !with_ld) || t->ld > INT32_MAX) return SBP_ERR_UNSUPPORTED;
    if (!is_sbp(s[0]) || !is_sbp(s[1])) return SBP_ERR_AXIS;
    for (int32_t a = 0; a < k0; ++a)
        for (int32_t b = 0; b < k1; ++b) {
            const Local l = local_of2(t->rows, t->cols, s, k0, k1, a, b);
            if (l.rows * l.cols == 0) continue;
            if (t->ld && l.cols > t->ld) return SBP_ERR_SHAPE;
            void* p = t->shard[a * k1 + b];
            if (!p) return SBP_ERR_NULL;
            if (reinterpret_cast<uintptr_t>(p) & 15u) return SBP_ERR_ALIGN;
        }
    return SBP_OK;
}
void spans_of2(const sbp_tensor_t* t, const sbp_t* s, int32_t k0, int32_t k1, std::vector<Span>& v) {
    for (int32_t a = 0; a < k0; ++a)
        for (int32_t b = 0; b < k1; ++b) {
            const Local l = local_of2(t->rows, t->cols, s, k0, k1, a, b);
            if (l.rows * l.cols == 0) continue;
            const uintptr_t bytes = (uintptr_t)((l.rows - 1) * pitch_of(t, l) + l.cols) * elem_bytes(t->dtype);
            const uintptr_t lo = reinterpret_cast<uintptr_t>(t->shard[a * k1 + b]);
            v.push_back({lo, lo + bytes});
        }
}

// outputs must be pairwise disjoint and disjoint from every input
int32_t check_alias(const std::vector<Span>& outs, const std::vector<Span>& ins) {
    for (size_t a = 0; a < outs.size(); ++a) {
        for (size_t b = a + 1; b < outs.size(); ++b)
            if (overlap(outs[a], outs[b])) return SBP_ERR_ALIAS;
        for (const Span& in : ins)
            if (overlap(outs[a], in)) return SBP_ERR_ALIAS;
    }
    return SBP_OK;
}

}  // namespace

extern "C" {

const char* sbp_strerror(int32_t status) {
    switch (status) {
        case SBP_OK: return "ok";
        case SBP_ERR_NULL: return "null descriptor, shard array or shard pointer";
        case SBP_ERR_K: return "k out of range";
        case SBP_ERR_SHAPE: return "bad or incompatible shape";
        case SBP_ERR_DTYPE: return "dtype not allowed here";
        case SBP_ERR_AXIS: return "not an SBP signature";
        case SBP_ERR_SIGNATURE: return "signature pair not valid for MatMul, or output signature is not the deduced one";
        case SBP_ERR_ALIAS: return "output buffer overlaps another buffer";
        case SBP_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case SBP_ERR_UNSUPPORTED: return "valid request without a kernel in this build";
        case SBP_ERR_LAUNCH: return "HIP launch failed";
        default: return "unknown status";
    }
}

int32_t sbp_probe_mfma(int32_t mode, int32_t iters, int32_t zero_operands, void* scratch, void* stream) {
    if (!scratch) return SBP_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(scratch) & 15u) return SBP_ERR_ALIGN;
    if (mode < 0 || mode > 8 || iters < 1 || iters > (1 << 24)) return SBP_ERR_UNSUPPORTED;
    return launch_probe_mfma(mode, iters, zero_operands ? 1 : 0, scratch, static_cast<hipStream_t>(stream));
}

int32_t sbp_probe_mfma_static(int32_t mode, int32_t iters, int32_t zero_operands, void* out, void* stream) {
    if (!out) return SBP_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(out) & 15u) return SBP_ERR_ALIGN;
    // modes 7 and 8 walk 1.5 GiB of caller memory: beyond what the library's own array holds
    if (mode < 0 || mode > 6 || iters < 1 || iters > (1 << 24)) return SBP_ERR_UNSUPPORTED;
    return launch_probe_mfma_static(mode, iters, zero_operands ? 1 : 0, out, static_cast<hipStream_t>(stream));
}

int32_t sbp_set_knob(int32_t knob, int32_t value) {
    if (knob == SBP_KNOB_GEMM_VARIANT && value >= 0 && value < 64) {
        g_gemm_variant.store(value);
        return SBP_OK;
    }
    if (knob == SBP_KNOB_TILE_ORDER && value >= 0 && value < 0x200) {
        set_tile_order(value);
        return SBP_OK;
    }
    if (knob == SBP_KNOB_BOX_REDUCE && (value == 0 || value == 1 || value == 2 || value == 4 || value == 8 || value == 16)) {
        set_box_reduce_variant(value);
        return SBP_OK;
    }
    return SBP_ERR_UNSUPPORTED;
}

int32_t sbp_infer_matmul(sbp_t sx, sbp_t sw, sbp_t* sy) {
    if (!sy) return SBP_ERR_NULL;
    if (!is_sbp(sx) || !is_sbp(sw)) return SBP_ERR_AXIS;
    // Table 1: the six valid rows, in the paper's order.
    if (sx == SBP_S(0) && sw == SBP_B) { *sy = SBP_S(0); return SBP_OK; }
    if (sx == SBP_B && sw == SBP_S(1)) { *sy = SBP_S(1); return SBP_OK; }
    if (sx == SBP_S(1) && sw == SBP_S(0)) { *sy = SBP_P_SUM; return SBP_OK; }
    if (sx == SBP_P_SUM && sw == SBP_B) { *sy = SBP_P_SUM; return SBP_OK; }
    if (sx == SBP_B && sw == SBP_P_SUM) { *sy = SBP_P_SUM; return SBP_OK; }
    if (sx == SBP_B && sw == SBP_B) { *sy = SBP_B; return SBP_OK; }
    return SBP_ERR_SIGNATURE;
}

int32_t sbp_local_shape(int64_t rows, int64_t cols, sbp_t s, int32_t k, int32_t i, int64_t* lr, int64_t* lc) {
    if (!lr || !lc) return SBP_ERR_NULL;
    if (k < 1 || k > SBP_MAX_K || i < 0 || i >= k) return SBP_ERR_K;
    if (rows < 0 || cols < 0) return SBP_ERR_SHAPE;
    if (!is_sbp(s)) return SBP_ERR_AXIS;
    const Local l = local_of(rows, cols, s, k, i);
    *lr = l.rows;
    *lc = l.cols;
    return SBP_OK;
}

// rowmax != nullptr: also reduce every stored row over the local columns into rowmax (P(max), [M,1] f32)
static int32_t matmul_impl(const sbp_tensor_t* x, sbp_t sx, const sbp_tensor_t* w, sbp_t sw, const sbp_tensor_t* y,
                           sbp_t sy, int32_t k, void* stream, int32_t epilogue, const sbp_tensor_t* rowmax) {
    if (k < 1 || k > SBP_MAX_K) return SBP_ERR_K;
    if (!x || !w || !y) return SBP_ERR_NULL;
    if (!is_sbp(sx) || !is_sbp(sw)) return SBP_ERR_AXIS;
    sbp_t deduced;
    int32_t st = sbp_infer_matmul(sx, sw, &deduced);
    if (st != SBP_OK) return st;
    if (sy == SBP_AUTO) sy = deduced;
    if (!is_sbp(sy)) return SBP_ERR_AXIS;
    if (sy != deduced) return SBP_ERR_SIGNATURE;
    if ((st = check_tensor(x, sx, k, true)) != SBP_OK) return st;
    if ((st = check_tensor(w, sw, k, true)) != SBP_OK) return st;
    if ((st = check_tensor(y, sy, k, true)) != SBP_OK) return st;
    if (x->cols != w->rows || y->rows != x->rows || y->cols != w->cols) return SBP_ERR_SHAPE;
    // a P(sum) operand is fp32; its partner may be fp32 or bf16 (rows 4 and 5 of Table 1 inside a bf16 graph)
    int32_t f32_operand = 0;
    if (is_partial(sx) && x->dtype != SBP_F32) return SBP_ERR_DTYPE;
    if (is_partial(sw) && w->dtype != SBP_F32) return SBP_ERR_DTYPE;
    if (x->dtype != w->dtype) {
        // fp32 next to bf16: the fp32 tensor is a P(sum) partial or the B tensor a reduced partial was boxed into
        if (x->dtype == SBP_F32 && (is_partial(sx) || sx == SBP_B) && sw == SBP_B) f32_operand = 1;
        else if (w->dtype == SBP_F32 && (is_partial(sw) || sw == SBP_B) && sx == SBP_B) f32_operand = 2;
        else return SBP_ERR_DTYPE;
    }
    const int32_t want_out = (is_partial(sy) || f32_operand) ? SBP_F32 : x->dtype;
    if (y->dtype != want_out) return SBP_ERR_DTYPE;
    if (y->trans != 0) return SBP_ERR_UNSUPPORTED;
    if (epilogue != SBP_EPI_NONE && epilogue != SBP_EPI_GELU) return SBP_ERR_UNSUPPORTED;
    if (epilogue == SBP_EPI_GELU && is_partial(sy)) return SBP_ERR_SIGNATURE;
    if (x->rows > INT32_MAX || x->cols > INT32_MAX || w->cols > INT32_MAX) return SBP_ERR_UNSUPPORTED;

    std::vector<Span> ins, outs;
    spans_of(x, sx, k, ins);
    spans_of(w, sw, k, ins);
    spans_of(y, sy, k, outs);
    if (rowmax) {
        if (sy != SBP_S(1)) return SBP_ERR_SIGNATURE;   // only a column-split result has partial row maxima
        if (epilogue != SBP_EPI_NONE) return SBP_ERR_UNSUPPORTED;
        if (!rowmax->shard) return SBP_ERR_NULL;
        if (rowmax->rows != y->rows || rowmax->cols != 1) return SBP_ERR_SHAPE;
        if (rowmax->dtype != SBP_F32) return SBP_ERR_DTYPE;
        if (rowmax->trans) return SBP_ERR_UNSUPPORTED;
        for (int32_t i = 0; i < k && y->rows > 0; ++i) {
            if (!rowmax->shard[i]) return SBP_ERR_NULL;
            if (reinterpret_cast<uintptr_t>(rowmax->shard[i]) & 15u) return SBP_ERR_ALIGN;
            const uintptr_t lo = reinterpret_cast<uintptr_t>(rowmax->shard[i]);
            outs.push_back({lo, lo + (uintptr_t)y->rows * 4});
        }
    }
    // (a B output written k times to one buffer would be k writers of the same bytes: refused as well)
    if ((st = check_alias(outs, ins)) != SBP_OK) return st;

    GemmPlan plan{};
    plan.groups = k;
    plan.in_dtype = f32_operand ? SBP_BF16 : x->dtype;
    plan.f32_operand = f32_operand;
    plan.out_dtype = y->dtype;
    plan.a_kc = x->trans ? 0 : 1;
    plan.b_kc = w->trans ? 1 : 0;
    plan.epilogue = epilogue;
    for (int32_t i = 0; i < k; ++i) {
        const Local lx = local_of(x->rows, x->cols, sx, k, i);
        const Local lw = local_of(w->rows, w->cols, sw, k, i);
        const Local ly = local_of(y->rows, y->cols, sy, k, i);
        if (lx.cols != lw.rows || ly.rows != lx.rows || ly.cols != lw.cols) return SBP_ERR_SHAPE;
        GemmShard& g = plan.s[i];
        g.a = x->shard[i];
        g.b = w->shard[i];
        g.c = y->shard[i];
        g.m = (int32_t)lx.rows;
        g.n = (int32_t)lw.cols;
        g.kk = (int32_t)lx.cols;
        g.lda = (int32_t)pitch_of(x, lx);
        g.ldb = (int32_t)pitch_of(w, lw);
        g.ldc = (int32_t)pitch_of(y, ly);
        g.rowmax = rowmax ? static_cast<float*>(rowmax->shard[i]) : nullptr;
    }
    if (!rowmax) return launch_gemm(plan, g_gemm_variant.load(), static_cast<hipStream_t>(stream));
    // fused where the kernel has it, else the product followed by the row reduction
    plan.epilogue = EPI_ROWMAX;
    st = launch_gemm(plan, g_gemm_variant.load(), static_cast<hipStream_t>(stream));
    if (st != SBP_ERR_UNSUPPORTED) return st;
    plan.epilogue = SBP_EPI_NONE;
    if ((st = launch_gemm(plan, g_gemm_variant.load(), static_cast<hipStream_t>(stream))) != SBP_OK) return st;
    RowStatPlan rs{};
    rs.rows = y->rows;
    rs.k = k;
    rs.dtype = y->dtype;
    for (int32_t i = 0; i < k; ++i) {
        rs.logits[i] = y->shard[i];
        rs.gmax[i] = nullptr;
        rs.out[i] = static_cast<float*>(rowmax->shard[i]);
        const Local ly = local_of(y->rows, y->cols, sy, k, i);
        rs.cols[i] = (int32_t)ly.cols;
        rs.ld[i] = (int32_t)pitch_of(y, ly);
    }
    return launch_row_stat(rs, false, static_cast<hipStream_t>(stream));
}

int32_t sbp_matmul_ex(const sbp_tensor_t* x, sbp_t sx, const sbp_tensor_t* w, sbp_t sw, const sbp_tensor_t* y,
                      sbp_t sy, int32_t k, void* stream, int32_t epilogue) {
    return matmul_impl(x, sx, w, sw, y, sy, k, stream, epilogue, nullptr);
}

int32_t sbp_matmul_rowmax(const sbp_tensor_t* x, sbp_t sx, const sbp_tensor_t* w, sbp_t sw, const sbp_tensor_t* y,
                          sbp_t sy, const sbp_tensor_t* rowmax, int32_t k, void* stream) {
    if (!rowmax) return SBP_ERR_NULL;
    return matmul_impl(x, sx, w, sw, y, sy, k, stream, SBP_EPI_NONE, rowmax);
}

int32_t sbp_matmul(const sbp_tensor_t* x, sbp_t sx, const sbp_tensor_t* w, sbp_t sw, const sbp_tensor_t* y,
                   sbp_t sy, int32_t k, void* stream) {
    return sbp_matmul_ex(x, sx, w, sw, y, sy, k, stream, SBP_EPI_NONE);
}

// launch = false: every check, nothing enqueued (the 2-D entry validates all its 1-D parts first)
// k_in = k_out: one device set; otherwise two disjoint placements
static int32_t boxing_impl(const sbp_tensor_t* in, sbp_t s_in, int32_t k_in, const sbp_tensor_t* out, sbp_t s_out,
                           int32_t k_out, void* stream, bool launch) {
    if (k_in < 1 || k_in > SBP_MAX_K || k_out < 1 || k_out > SBP_MAX_K) return SBP_ERR_K;
    if (!in || !out) return SBP_ERR_NULL;
    int32_t st;
    if ((st = check_tensor(in, s_in, k_in)) != SBP_OK) return st;
    if ((st = check_tensor(out, s_out, k_out)) != SBP_OK) return st;
    if (in->rows != out->rows || in->cols != out->cols) return SBP_ERR_SHAPE;
    if (in->dtype != out->dtype) return SBP_ERR_DTYPE;
    if ((is_partial(s_in) || is_partial(s_out)) && in->dtype != SBP_F32) return SBP_ERR_DTYPE;
    if (in->trans || out->trans) return SBP_ERR_UNSUPPORTED;
    if (is_partial(s_in) && is_partial(s_out) && s_in != s_out) return SBP_ERR_SIGNATURE;

    std::vector<Span> ins, outs;
    spans_of(in, s_in, k_in, ins);
    spans_of(out, s_out, k_out, outs);
    if ((st = check_alias(outs, ins)) != SBP_OK) return st;

    BoxPlan plan{};
    plan.rows = in->rows;
    plan.cols = in->cols;
    plan.k = k_in;
    plan.k_out = k_out;
    plan.sbp_in = s_in;
    plan.sbp_out = s_out;
    plan.elem_bytes = elem_bytes(in->dtype);
    for (int32_t i = 0; i < k_in; ++i) plan.src[i] = in->shard[i];
    for (int32_t i = 0; i < k_out; ++i) plan.dst[i] = out->shard[i];
    return launch ? launch_boxing(plan, static_cast<hipStream_t>(stream)) : SBP_OK;
}

int32_t sbp_boxing(const sbp_tensor_t* in, sbp_t s_in, const sbp_tensor_t* out, sbp_t s_out, int32_t k,
                   void* stream) {
    return boxing_impl(in, s_in, k, out, s_out, k, stream, true);
}

int32_t sbp_boxing_across(const sbp_tensor_t* in, sbp_t s_in, int32_t k_in, const sbp_tensor_t* out, sbp_t s_out,
                          int32_t k_out, void* stream) {
    return boxing_impl(in, s_in, k_in, out, s_out, k_out, stream, true);
}

int32_t sbp_boxing_cast(const sbp_tensor_t* in, sbp_t s_in, const sbp_tensor_t* out, sbp_t s_out, int32_t k,
                        void* stream) {
    if (k < 1 || k > SBP_MAX_K) return SBP_ERR_K;
    if (!in || !out) return SBP_ERR_NULL;
    int32_t st;
    if ((st = check_tensor(in, s_in, k)) != SBP_OK) return st;
    if ((st = check_tensor(out, s_out, k)) != SBP_OK) return st;
    if (in->rows != out->rows || in->cols != out->cols) return SBP_ERR_SHAPE;
    if (in->trans || out->trans) return SBP_ERR_UNSUPPORTED;
    const bool s_src = s_in == SBP_S(0) || s_in == SBP_S(1), s_dst = s_out == SBP_S(0) || s_out == SBP_S(1);
    const bool forward = s_src && s_out == SBP_B, backward = s_in == SBP_P_SUM && s_dst;
    if (!forward && !backward) return SBP_ERR_SIGNATURE;
    if (forward && (in->dtype != SBP_F32 || out->dtype != SBP_BF16)) return SBP_ERR_DTYPE;
    if (backward && (in->dtype != SBP_BF16 || out->dtype != SBP_F32)) return SBP_ERR_DTYPE;

    std::vector<Span> ins, outs;
    spans_of(in, s_in, k, ins);
    spans_of(out, s_out, k, outs);
    if ((st = check_alias(outs, ins)) != SBP_OK) return st;

    BoxPlan plan{};
    plan.rows = in->rows;
    plan.cols = in->cols;
    plan.k = plan.k_out = k;
    plan.sbp_in = s_in;
    plan.sbp_out = s_out;
    plan.elem_bytes = 0;
    for (int32_t i = 0; i < k; ++i) {
        plan.src[i] = in->shard[i];
        plan.dst[i] = out->shard[i];
    }
    return launch_boxing_cast(plan, static_cast<hipStream_t>(stream));
}

int32_t sbp_infer_matmul_2d(const sbp_t* sx, const sbp_t* sw, sbp_t* sy) {
    if (!sx || !sw || !sy) return SBP_ERR_NULL;
    sbp_t y[2];
    for (int d = 0; d < 2; ++d) {
        const int32_t st = sbp_infer_matmul(sx[d], sw[d], &y[d]);
        if (st != SBP_OK) return st;
    }
    sy[0] = y[0];
    sy[1] = y[1];
    return SBP_OK;
}

int32_t sbp_local_shape_2d(int64_t rows, int64_t cols, const sbp_t* s, int32_t k0, int32_t k1, int32_t a, int32_t b,
                           int64_t* lr, int64_t* lc) {
    if (!s || !lr || !lc) return SBP_ERR_NULL;
    int32_t st;
    if ((st = check_grid(k0, k1)) != SBP_OK) return st;
    if (a < 0 || a >= k0 || b < 0 || b >= k1) return SBP_ERR_K;
    if (rows < 0 || cols < 0) return SBP_ERR_SHAPE;
    if (!is_sbp(s[0]) || !is_sbp(s[1])) return SBP_ERR_AXIS;
    const Local l = local_of2(rows, cols, s, k0, k1, a, b);
    *lr = l.rows;
    *lc = l.cols;
    return SBP_OK;
}

int32_t sbp_matmul_2d(const sbp_tensor_t* x, const sbp_t* sx, const sbp_tensor_t* w, const sbp_t* sw,
                      const sbp_tensor_t* y, const sbp_t* sy_in, int32_t k0, int32_t k1, void* stream) {
    int32_t st;
    if ((st = check_grid(k0, k1)) != SBP_OK) return st;
    if (!x || !w || !y || !sx || !sw) return SBP_ERR_NULL;
    sbp_t sy[2];
    if ((st = sbp_infer_matmul_2d(sx, sw, sy)) != SBP_OK) return st;
    if (sy_in)
        for (int d = 0; d < 2; ++d) {
            if (sy_in[d] == SBP_AUTO) continue;
            if (!is_sbp(sy_in[d])) return SBP_ERR_AXIS;
            if (sy_in[d] != sy[d]) return SBP_ERR_SIGNATURE;
        }
    if ((st = check_tensor2(x, sx, k0, k1, true)) != SBP_OK) return st;
    if ((st = check_tensor2(w, sw, k0, k1, true)) != SBP_OK) return st;
    if ((st = check_tensor2(y, sy, k0, k1, true)) != SBP_OK) return st;
    if (x->cols != w->rows || y->rows != x->rows || y->cols != w->cols) return SBP_ERR_SHAPE;
    const bool px = is_partial(sx[0]) || is_partial(sx[1]), pw = is_partial(sw[0]) || is_partial(sw[1]);
    const bool py = is_partial(sy[0]) || is_partial(sy[1]);
    int32_t f32_operand = 0;
    if (px && x->dtype != SBP_F32) return SBP_ERR_DTYPE;
    if (pw && w->dtype != SBP_F32) return SBP_ERR_DTYPE;
    if (x->dtype != w->dtype) {
        if (px && x->dtype == SBP_F32) f32_operand = 1;
        else if (pw && w->dtype == SBP_F32) f32_operand = 2;
        else return SBP_ERR_DTYPE;
    }
    if (y->dtype != ((py || f32_operand) ? SBP_F32 : x->dtype)) return SBP_ERR_DTYPE;
    if (x->rows > INT32_MAX || x->cols > INT32_MAX || w->cols > INT32_MAX) return SBP_ERR_UNSUPPORTED;

    std::vector<Span> ins, outs;
    spans_of2(x, sx, k0, k1, ins);
    spans_of2(w, sw, k0, k1, ins);
    spans_of2(y, sy, k0, k1, outs);
    if ((st = check_alias(outs, ins)) != SBP_OK) return st;

    GemmPlan plan{};
    plan.groups = k0 * k1;
    plan.in_dtype = f32_operand ? SBP_BF16 : x->dtype;
    plan.f32_operand = f32_operand;
    plan.out_dtype = y->dtype;
    plan.a_kc = 1;
    plan.b_kc = 0;
    plan.epilogue = SBP_EPI_NONE;
    for (int32_t a = 0; a < k0; ++a)
        for (int32_t b = 0; b < k1; ++b) {
            const Local lx = local_of2(x->rows, x->cols, sx, k0, k1, a, b);
            const Local lw = local_of2(w->rows, w->cols, sw, k0, k1, a, b);
            const Local ly = local_of2(y->rows, y->cols, sy, k0, k1, a, b);
            if (lx.cols != lw.rows || ly.rows != lx.rows || ly.cols != lw.cols) return SBP_ERR_SHAPE;
            GemmShard& g = plan.s[a * k1 + b];
            g.a = x->shard[a * k1 + b];
            g.b = w->shard[a * k1 + b];
            g.c = y->shard[a * k1 + b];
            g.m = (int32_t)lx.rows;
            g.n = (int32_t)lw.cols;
            g.kk = (int32_t)lx.cols;
            g.lda = (int32_t)pitch_of(x, lx);
            g.ldb = (int32_t)pitch_of(w, lw);
            g.ldc = (int32_t)pitch_of(y, ly);
        }
    return launch_gemm(plan, g_gemm_variant.load(), static_cast<hipStream_t>(stream));
}

int32_t sbp_boxing_2d(const sbp_tensor_t* in, const sbp_t* s_in, const sbp_tensor_t* out, const sbp_t* s_out,
                      int32_t k0, int32_t k1, void* stream) {
    int32_t st;
    if ((st = check_grid(k0, k1)) != SBP_OK) return st;
    if (!in || !out || !s_in || !s_out) return SBP_ERR_NULL;
    if ((st = check_tensor2(in, s_in, k0, k1)) != SBP_OK) return st;
    if ((st = check_tensor2(out, s_out, k0, k1)) != SBP_OK) return st;
    if (in->rows != out->rows || in->cols != out->cols) return SBP_ERR_SHAPE;
    if (in->dtype != out->dtype) return SBP_ERR_DTYPE;
    const bool inner = s_in[0] == s_out[0];
    if (!inner && s_in[1] != s_out[1]) return SBP_ERR_UNSUPPORTED;   // one position at a time
    const sbp_t keep = inner ? s_in[0] : s_in[1];
    if (is_partial(keep) && in->dtype != SBP_F32) return SBP_ERR_DTYPE;
    // outer conversion with an inner split: the devices of inner index b hold slice b of the tensor
    // only if the conversion does not touch the axis the inner position splits
    if (!inner && (keep == SBP_S(0) || keep == SBP_S(1)) && (s_in[0] == keep || s_out[0] == keep)) return SBP_ERR_UNSUPPORTED;
    // (outer, inner) stands for outer-op over the groups of (inner-op over a group's devices): an outer partial
    // reduced device by device underneath an inner partial of the OTHER operation would swap the two reductions,
    // and sum and max do not commute
    if (!inner && is_partial(keep) && is_partial(s_in[0]) && s_in[0] != keep) return SBP_ERR_UNSUPPORTED;

    std::vector<Span> ins, outs;
    spans_of2(in, s_in, k0, k1, ins);
    spans_of2(out, s_out, k0, k1, outs);
    if ((st = check_alias(outs, ins)) != SBP_OK) return st;

    const int32_t parts = inner ? k0 : k1, kk = inner ? k1 : k0;
    std::vector<void*> pin((size_t)parts * kk), pout((size_t)parts * kk);
    std::vector<sbp_tensor_t> tin(parts), tout(parts);
    for (int32_t g = 0; g < parts; ++g) {
        for (int32_t i = 0; i < kk; ++i) {
            const int32_t dev = inner ? g * k1 + i : i * k1 + g;
            pin[(size_t)g * kk + i] = in->shard[dev];
            pout[(size_t)g * kk + i] = out->shard[dev];
        }
        // the tensor this group of devices holds between them
        const Local l = inner ? local_of(in->rows, in->cols, keep, k0, g) : local_of(in->rows, in->cols, keep, k1, g);
        tin[g] = {&pin[(size_t)g * kk], l.rows, l.cols, in->dtype, 0};
        tout[g] = {&pout[(size_t)g * kk], l.rows, l.cols, out->dtype, 0};
    }
    const sbp_t a = inner ? s_in[1] : s_in[0], b = inner ? s_out[1] : s_out[0];
    for (int32_t g = 0; g < parts; ++g) {   // validate every part before anything is enqueued
        if (tin[g].rows * tin[g].cols == 0) continue;
        if ((st = boxing_impl(&tin[g], a, kk, &tout[g], b, kk, stream, false)) != SBP_OK) return st;
    }
    // Reductions of equally shaped parts go out as ONE launch (pin and pout already hold the pointers part by part):
    // two half-size kernels one after the other leave the memory system idle at the seam.
    bool same = parts > 1 && is_partial(a) && tin[0].rows * tin[0].cols > 0;
    for (int32_t g = 1; g < parts && same; ++g) same = tin[g].rows == tin[0].rows && tin[g].cols == tin[0].cols;
    if (same) {
        BoxPlan plan{};
        plan.rows = tin[0].rows;
        plan.cols = tin[0].cols;
        plan.k = plan.k_out = kk;
        plan.sbp_in = a;
        plan.sbp_out = b;
        plan.elem_bytes = elem_bytes(in->dtype);
        plan.batch = parts;
        for (size_t i = 0; i < pin.size(); ++i) {
            plan.src[i] = pin[i];
            plan.dst[i] = pout[i];
        }
        st = launch_boxing(plan, static_cast<hipStream_t>(stream));
        if (st != SBP_ERR_UNSUPPORTED) return st;   // unsupported as a batch: nothing was enqueued, go part by part
    }
    for (int32_t g = 0; g < parts; ++g) {
        if (tin[g].rows * tin[g].cols == 0) continue;
        if ((st = boxing_impl(&tin[g], a, kk, &tout[g], b, kk, stream, true)) != SBP_OK) return st;
    }
    return SBP_OK;
}

static int32_t row_stat(const sbp_tensor_t* logits, sbp_t sl, const sbp_tensor_t* gmax, const sbp_tensor_t* out,
                        int32_t k, void* stream, bool sumexp) {
    if (k < 1 || k > SBP_MAX_K) return SBP_ERR_K;
    if (!logits || !out || (sumexp && !gmax)) return SBP_ERR_NULL;
    int32_t st;
    if ((st = check_tensor(logits, sl, k, true)) != SBP_OK) return st;
    if (is_partial(sl)) return SBP_ERR_SIGNATURE;  // row statistics of an un-reduced partial are meaningless
    if (sl != SBP_S(1)) return SBP_ERR_UNSUPPORTED;  // only the model-parallel case yields partial vectors
    const sbp_t s_out = sumexp ? SBP_P_SUM : SBP_P_MAX;
    if ((st = check_tensor(out, s_out, k)) != SBP_OK) return st;
    if (sumexp && (st = check_tensor(gmax, SBP_B, k)) != SBP_OK) return st;
    if (out->rows != logits->rows || out->cols != 1 || out->dtype != SBP_F32) return SBP_ERR_SHAPE;
    if (sumexp && (gmax->rows != logits->rows || gmax->cols != 1 || gmax->dtype != SBP_F32)) return SBP_ERR_SHAPE;
    if (logits->trans || out->trans || (sumexp && gmax->trans)) return SBP_ERR_UNSUPPORTED;
    if (logits->cols > INT32_MAX) return SBP_ERR_UNSUPPORTED;

    std::vector<Span> ins, outs;
    spans_of(logits, sl, k, ins);
    if (sumexp) spans_of(gmax, SBP_B, k, ins);
    spans_of(out, s_out, k, outs);
    if ((st = check_alias(outs, ins)) != SBP_OK) return st;

    RowStatPlan plan{};
    plan.rows = logits->rows;
    plan.k = k;
    plan.dtype = logits->dtype;
    for (int32_t i = 0; i < k; ++i) {
        plan.logits[i] = logits->shard[i];
        plan.gmax[i] = sumexp ? static_cast<const float*>(gmax->shard[i]) : nullptr;
        plan.out[i] = static_cast<float*>(out->shard[i]);
        const Local l = local_of(logits->rows, logits->cols, sl, k, i);
        plan.cols[i] = (int32_t)l.cols;
        plan.ld[i] = (int32_t)pitch_of(logits, l);
    }
    return launch_row_stat(plan, sumexp, static_cast<hipStream_t>(stream));
}

// labels: [R,1] SBP_I32, B (one device pointer per logical device; copies may share a buffer)
static int32_t check_vector(const sbp_tensor_t* t, int64_t rows, int32_t dtype, int32_t k) {
    if (!t || !t->shard) return SBP_ERR_NULL;
    if (t->rows != rows || t->cols != 1) return SBP_ERR_SHAPE;
    if (t->dtype != dtype) return SBP_ERR_DTYPE;
    if (t->trans) return SBP_ERR_UNSUPPORTED;
    for (int32_t i = 0; i < k && rows > 0; ++i) {
        if (!t->shard[i]) return SBP_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(t->shard[i]) & 15u) return SBP_ERR_ALIGN;
    }
    return SBP_OK;
}
static void spans_of_vector(const sbp_tensor_t* t, int32_t k, std::vector<Span>& v) {
    for (int32_t i = 0; i < k; ++i) {
        const uintptr_t lo = reinterpret_cast<uintptr_t>(t->shard[i]);
        if (t->rows) v.push_back({lo, lo + (uintptr_t)t->rows * 4});
    }
}

static int32_t xent(const sbp_tensor_t* logits, sbp_t sl, const sbp_tensor_t* labels, const sbp_tensor_t* gmax,
                    const sbp_tensor_t* denom, const sbp_tensor_t* grad, const sbp_tensor_t* out, int32_t k, void* stream) {
    if (k < 1 || k > SBP_MAX_K) return SBP_ERR_K;
    if (!logits || !labels || !gmax || !denom || !out) return SBP_ERR_NULL;
    int32_t st;
    if ((st = check_tensor(logits, sl, k, true)) != SBP_OK) return st;
    if (sl != SBP_S(1)) return is_partial(sl) ? SBP_ERR_SIGNATURE : SBP_ERR_UNSUPPORTED;
    if (k > XENT_MAX_K) return SBP_ERR_UNSUPPORTED;
    if (logits->trans) return SBP_ERR_UNSUPPORTED;
    if (logits->cols > INT32_MAX || logits->rows > INT32_MAX) return SBP_ERR_UNSUPPORTED;
    const int64_t R = logits->rows;
    if ((st = check_vector(labels, R, SBP_I32, k)) != SBP_OK) return st;
    if ((st = check_vector(gmax, R, SBP_F32, k)) != SBP_OK) return st;
    if ((st = check_vector(denom, R, SBP_F32, k)) != SBP_OK) return st;
    if (grad && (st = check_vector(grad, R, SBP_F32, k)) != SBP_OK) return st;
    std::vector<Span> ins, outs;
    spans_of(logits, sl, k, ins);
    spans_of_vector(labels, k, ins);
    spans_of_vector(gmax, k, ins);
    spans_of_vector(denom, k, ins);
    if (grad) {
        spans_of_vector(grad, k, ins);
        if ((st = check_tensor(out, SBP_S(1), k, true)) != SBP_OK) return st;
        if (out->rows != R || out->cols != logits->cols || out->dtype != logits->dtype || out->trans) return SBP_ERR_SHAPE;
        spans_of(out, SBP_S(1), k, outs);
    } else {
        if ((st = check_vector(out, R, SBP_F32, k)) != SBP_OK) return st;
        spans_of_vector(out, k, outs);
    }
    if ((st = check_alias(outs, ins)) != SBP_OK) return st;

    XentPlan plan{};
    plan.rows = R;
    plan.total_cols = (int32_t)logits->cols;
    plan.k = k;
    plan.dtype = logits->dtype;
    for (int32_t i = 0; i < k; ++i) {
        plan.logits[i] = logits->shard[i];
        plan.labels[i] = static_cast<const int32_t*>(labels->shard[i]);
        plan.gmax[i] = static_cast<const float*>(gmax->shard[i]);
        plan.denom[i] = static_cast<const float*>(denom->shard[i]);
        plan.grad[i] = grad ? static_cast<const float*>(grad->shard[i]) : nullptr;
        plan.out[i] = out->shard[i];
        plan.cols[i] = (int32_t)split_len(logits->cols, k, i);
        plan.ld[i] = logits->ld ? (int32_t)logits->ld : plan.cols[i];
        plan.ld_out[i] = (grad && out->ld) ? (int32_t)out->ld : plan.cols[i];
        plan.begin[i] = (int32_t)split_begin(logits->cols, k, i);
    }
    return grad ? launch_xent_grad(plan, static_cast<hipStream_t>(stream)) : launch_xent_loss(plan, static_cast<hipStream_t>(stream));
}

int32_t sbp_xent_loss(const sbp_tensor_t* logits, sbp_t sl, const sbp_tensor_t* labels, const sbp_tensor_t* gmax,
                      const sbp_tensor_t* denom, const sbp_tensor_t* loss, int32_t k, void* stream) {
    return xent(logits, sl, labels, gmax, denom, nullptr, loss, k, stream);
}

int32_t sbp_xent_grad(const sbp_tensor_t* logits, sbp_t sl, const sbp_tensor_t* labels, const sbp_tensor_t* gmax,
                      const sbp_tensor_t* denom, const sbp_tensor_t* grad, const sbp_tensor_t* dlogits, int32_t k,
                      void* stream) {
    if (!grad) return SBP_ERR_NULL;
    return xent(logits, sl, labels, gmax, denom, grad, dlogits, k, stream);
}

int32_t sbp_row_max(const sbp_tensor_t* logits, sbp_t sl, const sbp_tensor_t* out, int32_t k, void* stream) {
    return row_stat(logits, sl, nullptr, out, k, stream, false);
}

int32_t sbp_row_sumexp(const sbp_tensor_t* logits, sbp_t sl, const sbp_tensor_t* gmax, const sbp_tensor_t* out,
                       int32_t k, void* stream) {
    return row_stat(logits, sl, gmax, out, k, stream, true);
}

}  // extern "C"
