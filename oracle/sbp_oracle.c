/*
 * CPU oracle for the SBP matmul + boxing path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the arithmetic half of the oracle (the layout half, scatter /
 * assemble / boxing, is numpy slicing in sbp_oracle.py).  Everything here is
 * the plain definition in double precision, one loop nest per function, no
 * blocking, no fusion.  It shares no code with the HIP library; only tests,
 * the smoke check and the bench's cpu_baseline leg may load it.
 *
 * What each function follows (OneFlow paper, arXiv 2110.15032):
 *   orc_split_range      Sec. 3.1, split "in a balanced manner"; the paper is
 *                        silent on uneven sizes, the reading taken here is
 *                        floor(n/k) everywhere plus one extra index on the
 *                        first (n mod k) shards.
 *   orc_matmul           Sec. 3.1, Y = XW for one local (or the logical) pair.
 *   orc_reduce_sum/max   Sec. 3.1, partial-value: the global tensor is the
 *                        element-wise reduction over all local tensors.
 *   orc_row_max/sumexp   Sec. 6.3.1, the two reductions inside the model-
 *                        parallel softmax (max, then sum of exp(l - max)).
 *   orc_gelu             not in the paper (the workload adds it); exact erf
 *                        form 0.5 x (1 + erf(x / sqrt 2)).
 *   orc_bf16_*           bfloat16 = top 16 bits of an IEEE binary32; rounding
 *                        is to nearest, ties to even, done ONCE from the
 *                        double value.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC sbp_oracle.c -o libsbp_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* shard i of k over an axis of length n owns indices [*begin, *begin + *len) */
void orc_split_range(int64_t n, int32_t k, int32_t i, int64_t* begin, int64_t* len) {
    int64_t q = n / k, r = n % k;
    *len = q + (i < r ? 1 : 0);
    *begin = (int64_t)i * q + (i < r ? i : r);
}

/* C[M,N] = A[M,K] * B[K,N], row-major, double accumulation, k ascending. */
void orc_matmul(const double* A, const double* B, double* C,
                int64_t M, int64_t K, int64_t N) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double* c = C + m * N;
        for (int64_t n = 0; n < N; ++n) c[n] = 0.0;
        for (int64_t kk = 0; kk < K; ++kk) {
            const double a = A[m * K + kk];
            const double* b = B + kk * N;
            for (int64_t n = 0; n < N; ++n) c[n] += a * b[n];
        }
    }
}

/* out[e] = parts[0][e] + parts[1][e] + ... + parts[k-1][e] */
void orc_reduce_sum(const double* const* parts, int32_t k, double* out, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        double s = 0.0;
        for (int32_t i = 0; i < k; ++i) s += parts[i][e];
        out[e] = s;
    }
}

/* max of two values under the reading taken for P(max) (the paper names the operation only): a NaN is
 * ignored next to a number, NaN results only when both are NaN; of +0 and -0 the first one stays. */
static double max_ignoring_nan(double s, double x) {
    if (s != s) return x;
    return x > s ? x : s;
}

/* out[e] = max_i parts[i][e] */
void orc_reduce_max(const double* const* parts, int32_t k, double* out, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        double s = parts[0][e];
        for (int32_t i = 1; i < k; ++i) s = max_ignoring_nan(s, parts[i][e]);
        out[e] = s;
    }
}

void orc_gelu(const double* x, double* y, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e)
        y[e] = 0.5 * x[e] * (1.0 + erf(x[e] / sqrt(2.0)));
}

/* m[r] = max_c L[r,c] */
void orc_row_max(const double* L, int64_t rows, int64_t cols, double* m) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double v = L[r * cols];
        for (int64_t c = 1; c < cols; ++c) v = max_ignoring_nan(v, L[r * cols + c]);
        m[r] = v;
    }
}

/* s[r] = sum_c exp(L[r,c] - m[r]) */
void orc_row_sumexp(const double* L, const double* m, int64_t rows, int64_t cols, double* s) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double v = 0.0;
        for (int64_t c = 0; c < cols; ++c) v += exp(L[r * cols + c] - m[r]);
        s[r] = v;
    }
}

/* Nearest bfloat16 (ties to even) of a double, as its 16-bit pattern.
 * A finite bf16 is +-(integer q < 2^8) * 2^(e-8) with the value's binary
 * exponent e clamped below at the smallest normal one (-126), so rounding is
 * "scale to that grid, rint (ties-to-even in the default mode), scale back". */
static uint16_t bf16_bits_from_f64(double x) {
    if (isnan(x)) return 0x7FC0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (isinf(a)) return sign | 0x7F80;
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);          /* a = f * 2^e, 0.5 <= f < 1  =>  2^(e-1) <= a < 2^e */
    int ex = e - 1;              /* unbiased exponent of a */
    if (ex < -126) ex = -126;    /* subnormal range shares the smallest normal's grid */
    double q = rint(ldexp(a, 7 - ex));   /* units of 2^(ex-7): 7 explicit mantissa bits */
    if (q >= 256.0) { q = 128.0; ex += 1; }   /* rounded up to the next binade */
    if (ex > 127) return sign | 0x7F80;       /* overflow -> infinity */
    uint32_t qi = (uint32_t)q;
    if (qi < 128) return sign | (uint16_t)qi;                 /* subnormal or zero */
    return sign | (uint16_t)(((uint32_t)(ex + 127) << 7) | (qi - 128));
}

void orc_bf16_from_f64(const double* x, uint16_t* out, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e) out[e] = bf16_bits_from_f64(x[e]);
}

/* exact widening: bf16 pattern -> the binary32 with those top 16 bits -> double */
void orc_bf16_to_f64(const uint16_t* in, double* out, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        uint32_t w = (uint32_t)in[e] << 16;
        float f;
        memcpy(&f, &w, 4);
        out[e] = (double)f;
    }
}
