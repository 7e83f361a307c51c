/*
 * CPU oracle: see xp_oracle.h.  TEST INFRASTRUCTURE ONLY.
 *
 * Each function is the operator's definition written as scalar loops.  Floating-point inputs
 * are widened to double before the multiply, products and sums are formed in double, k ascending.
 */
#include "xp_oracle.h"

#include <stddef.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double widen(const void *base, int type, int64_t idx)
{
    if (type == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else {
        /* bf16 is the upper half of an fp32: shift the bits up, the lower 16 are zero */
        uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &u, sizeof f);
        return (double)f;
    }
}

static inline int64_t at(int layout, int64_t i, int64_t j, int64_t ld)
{
    return layout == ORACLE_ROW ? i * ld + j : i + j * ld;
}

static int bad_type(int t) { return t != ORACLE_F32 && t != ORACLE_BF16; }
static int bad_layout(int l) { return l != ORACLE_ROW && l != ORACLE_COL; }

/* Not arithmetic: caps the threads of the loops below (timing the oracle on one core). n <= 0 restores the default. */
void oracle_set_num_threads(int n)
{
    static int initial = 0;
    if (initial == 0) initial = omp_get_max_threads();
    omp_set_num_threads(n > 0 ? n : initial);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int oracle_gemm_float(int64_t M, int64_t N, int64_t K, double alpha,
                      const void *A, int a_type, int a_layout, int64_t lda,
                      const void *B, int b_type, int b_layout, int64_t ldb,
                      double beta, const float *C0, int c_layout, int64_t ldc,
                      double *ref)
{
    if (M < 0 || N < 0 || K < 0) return 1;
    if (bad_type(a_type) || bad_type(b_type)) return 2;
    if (bad_layout(a_layout) || bad_layout(b_layout) || bad_layout(c_layout)) return 3;
    if (M == 0 || N == 0) return 0;
    if (!ref || (K > 0 && (!A || !B)) || (beta != 0.0 && !C0)) return 4;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = widen(A, a_type, at(a_layout, i, k, lda));
                double b = widen(B, b_type, at(b_layout, k, j, ldb));
                acc += a * b;
            }
            double r = alpha * acc;
            if (beta != 0.0) r += beta * (double)C0[at(c_layout, i, j, ldc)];
            ref[i * N + j] = r;
        }
    }
    return 0;
}

int oracle_gemm_i8(int64_t M, int64_t N, int64_t K,
                   const int8_t *A, int a_layout, int64_t lda,
                   const int8_t *B, int b_layout, int64_t ldb,
                   int32_t *ref)
{
    if (M < 0 || N < 0 || K < 0) return 1;
    if (bad_layout(a_layout) || bad_layout(b_layout)) return 3;
    if (M == 0 || N == 0) return 0;
    if (!ref || (K > 0 && (!A || !B))) return 4;

    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) {
                acc += (int64_t)A[at(a_layout, i, k, lda)] * (int64_t)B[at(b_layout, k, j, ldb)];
            }
            if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
            ref[i * N + j] = (int32_t)acc;
        }
    }
    return overflow ? 100 : 0;
}

int oracle_gemm_float_batched(int64_t batch, int64_t M, int64_t N, int64_t K, double alpha,
                              const void *A, int a_type, int a_layout, int64_t lda, int64_t strideA,
                              const void *B, int b_type, int b_layout, int64_t ldb, int64_t strideB,
                              double beta, const float *C0, int c_layout, int64_t ldc, int64_t strideC,
                              double *ref)
{
    if (batch < 0) return 1;
    if (bad_type(a_type) || bad_type(b_type)) return 2;
    const int64_t a_sz = a_type == ORACLE_F32 ? 4 : 2;
    const int64_t b_sz = b_type == ORACLE_F32 ? 4 : 2;
    for (int64_t b = 0; b < batch; ++b) {
        const char *Ab = A ? (const char *)A + b * strideA * a_sz : NULL;
        const char *Bb = B ? (const char *)B + b * strideB * b_sz : NULL;
        const float *Cb = C0 ? C0 + b * strideC : NULL;
        int rc = oracle_gemm_float(M, N, K, alpha, Ab, a_type, a_layout, lda,
                                   Bb, b_type, b_layout, ldb, beta, Cb, c_layout, ldc,
                                   ref ? ref + b * M * N : NULL);
        if (rc) return rc;
    }
    return 0;
}

int oracle_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                       int64_t R, int64_t S, int64_t stride_h, int64_t stride_w,
                       int64_t pad_h, int64_t pad_w,
                       const void *input, int in_type,
                       const void *filter, int w_type, int w_layout,
                       double *ref)
{
    if (N < 0 || H < 0 || W < 0 || Cin < 0 || Cout < 0 || R <= 0 || S <= 0) return 1;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return 1;
    if (bad_type(in_type) || bad_type(w_type)) return 2;
    if (w_layout != ORACLE_KRSC && w_layout != ORACLE_RSCK) return 3;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return 0;      /* empty output */
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1;
    const int64_t Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N == 0 || Cout == 0) return 0;
    if (!ref || (Cin > 0 && (!input || !filter))) return 4;

#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t p = 0; p < P; ++p) {
            for (int64_t q = 0; q < Q; ++q) {
                for (int64_t k = 0; k < Cout; ++k) {
                    double acc = 0.0;
                    for (int64_t r = 0; r < R; ++r) {
                        const int64_t h = p * stride_h + r - pad_h;
                        if (h < 0 || h >= H) continue;          /* zero padding: term is 0 */
                        for (int64_t s = 0; s < S; ++s) {
                            const int64_t w = q * stride_w + s - pad_w;
                            if (w < 0 || w >= W) continue;
                            for (int64_t c = 0; c < Cin; ++c) {
                                const int64_t wi = w_layout == ORACLE_KRSC
                                    ? ((k * R + r) * S + s) * Cin + c
                                    : ((r * S + s) * Cin + c) * Cout + k;
                                acc += widen(input, in_type, ((n * H + h) * W + w) * Cin + c)
                                     * widen(filter, w_type, wi);
                            }
                        }
                    }
                    ref[((n * P + p) * Q + q) * Cout + k] = acc;
                }
            }
        }
    }
    return 0;
}

/* Scaled dot-product attention without a mask: the scores of one query against every key, a
 * softmax over the keys, the weighted sum of the value rows.  The largest score is subtracted
 * before exponentiation (this does not change the quotient; it keeps exp() in range). */
int oracle_attention(int64_t batch, int64_t Lq, int64_t Lk, int64_t d, int64_t dv, double scale,
                     const void *Q, int q_type, int64_t ldq, int64_t strideQ,
                     const void *K, int k_type, int64_t ldk, int64_t strideK,
                     const void *V, int v_type, int64_t ldv, int64_t strideV,
                     double *ref)
{
    if (batch < 0 || Lq < 0 || Lk <= 0 || d < 0 || dv < 0) return 1;
    if (bad_type(q_type) || bad_type(k_type) || bad_type(v_type)) return 2;
    if (ldq < d || ldk < d || ldv < dv) return 3;
    if (batch == 0 || Lq == 0 || dv == 0) return 0;
    if (!ref || !V || (d > 0 && (!Q || !K))) return 4;

    int failed = 0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t i = 0; i < Lq; ++i) {
            double *w = (double *)malloc((size_t)Lk * sizeof(double));
            if (!w) {
#pragma omp atomic write
                failed = 1;
                continue;
            }
            double top = -INFINITY;
            for (int64_t j = 0; j < Lk; ++j) {
                double dot = 0.0;
                for (int64_t c = 0; c < d; ++c)
                    dot += widen(Q, q_type, b * strideQ + i * ldq + c) * widen(K, k_type, b * strideK + j * ldk + c);
                w[j] = scale * dot;
                if (w[j] > top) top = w[j];
            }
            double total = 0.0;
            for (int64_t j = 0; j < Lk; ++j) {
                w[j] = exp(w[j] - top);
                total += w[j];
            }
            for (int64_t x = 0; x < dv; ++x) {
                double acc = 0.0;
                for (int64_t j = 0; j < Lk; ++j)
                    acc += (w[j] / total) * widen(V, v_type, b * strideV + j * ldv + x);
                ref[(b * Lq + i) * dv + x] = acc;
            }
            free(w);
        }
    }
    return failed ? 5 : 0;
}

/* ---- row-wise operators over the last dimension: x is rows x cols with row pitch ldx ---- */

int oracle_softmax(int64_t rows, int64_t cols, const void *x, int x_type, int64_t ldx, double *ref)
{
    if (rows < 0 || cols < 0 || ldx < cols) return 1;
    if (bad_type(x_type)) return 2;
    if (rows == 0 || cols == 0) return 0;
    if (!x || !ref) return 4;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double top = -INFINITY, total = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            const double v = widen(x, x_type, i * ldx + j);
            if (v > top) top = v;
        }
        for (int64_t j = 0; j < cols; ++j) {
            ref[i * cols + j] = exp(widen(x, x_type, i * ldx + j) - top);
            total += ref[i * cols + j];
        }
        for (int64_t j = 0; j < cols; ++j) ref[i * cols + j] /= total;
    }
    return 0;
}

/* gamma and beta have the element type of x; NULL stands for all ones / all zeros */
int oracle_layernorm(int64_t rows, int64_t cols, const void *x, int x_type, int64_t ldx,
                     const void *gamma, const void *beta, double eps, double *ref)
{
    if (rows < 0 || cols < 0 || ldx < cols) return 1;
    if (bad_type(x_type)) return 2;
    if (rows == 0 || cols == 0) return 0;
    if (!x || !ref) return 4;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double mean = 0.0, var = 0.0;
        for (int64_t j = 0; j < cols; ++j) mean += widen(x, x_type, i * ldx + j);
        mean /= (double)cols;
        for (int64_t j = 0; j < cols; ++j) {
            const double d = widen(x, x_type, i * ldx + j) - mean;
            var += d * d;
        }
        var /= (double)cols;                                  /* the biased (population) variance */
        const double rstd = 1.0 / sqrt(var + eps);
        for (int64_t j = 0; j < cols; ++j) {
            const double g = gamma ? widen(gamma, x_type, j) : 1.0, b = beta ? widen(beta, x_type, j) : 0.0;
            ref[i * cols + j] = (widen(x, x_type, i * ldx + j) - mean) * rstd * g + b;
        }
    }
    return 0;
}

int oracle_rmsnorm(int64_t rows, int64_t cols, const void *x, int x_type, int64_t ldx,
                   const void *gamma, double eps, double *ref)
{
    if (rows < 0 || cols < 0 || ldx < cols) return 1;
    if (bad_type(x_type)) return 2;
    if (rows == 0 || cols == 0) return 0;
    if (!x || !ref) return 4;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double ms = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            const double v = widen(x, x_type, i * ldx + j);
            ms += v * v;
        }
        ms /= (double)cols;
        const double r = 1.0 / sqrt(ms + eps);
        for (int64_t j = 0; j < cols; ++j)
            ref[i * cols + j] = widen(x, x_type, i * ldx + j) * r * (gamma ? widen(gamma, x_type, j) : 1.0);
    }
    return 0;
}

/* ---- element-wise operators on n elements ---- */

int oracle_unary(int op, int64_t n, const void *x, int x_type, double *ref)
{
    if (n < 0) return 1;
    if (bad_type(x_type)) return 2;
    if (op < ORACLE_RELU || op > ORACLE_SIGN) return 3;
    if (n == 0) return 0;
    if (!x || !ref) return 4;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const double v = widen(x, x_type, i);
        double y;
        switch (op) {
        case ORACLE_RELU: y = v > 0.0 ? v : 0.0; break;
        case ORACLE_GELU: y = 0.5 * v * (1.0 + erf(v / sqrt(2.0))); break;
        case ORACLE_SIGMOID: y = 1.0 / (1.0 + exp(-v)); break;
        default: y = v > 0.0 ? 1.0 : (v < 0.0 ? -1.0 : 0.0); break;
        }
        ref[i] = y;
    }
    return 0;
}

int oracle_add(int64_t n, const void *a, const void *b, int type, double *ref)
{
    if (n < 0) return 1;
    if (bad_type(type)) return 2;
    if (n == 0) return 0;
    if (!a || !b || !ref) return 4;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) ref[i] = widen(a, type, i) + widen(b, type, i);
    return 0;
}

/* ---- 2-D pooling, NHWC.  Window positions outside the image do not take part: the maximum and
 * minimum are over the positions inside, the sum adds nothing for them, and the average divides by
 * the number of positions inside.  A window with no position inside gives 0. ---- */
int oracle_pool2d_nhwc(int op, int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                       int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                       const void *x, int x_type, double *ref)
{
    if (N < 0 || H < 0 || W < 0 || C < 0 || R <= 0 || S <= 0) return 1;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return 1;
    if (bad_type(x_type)) return 2;
    if (op < ORACLE_POOL_MAX || op > ORACLE_POOL_SUM) return 3;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return 0;
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N == 0 || C == 0) return 0;
    if (!x || !ref) return 4;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t c = 0; c < C; ++c) {
                    double acc = 0.0;
                    int64_t inside = 0;
                    for (int64_t r = 0; r < R; ++r) {
                        const int64_t h = p * stride_h + r - pad_h;
                        if (h < 0 || h >= H) continue;
                        for (int64_t s = 0; s < S; ++s) {
                            const int64_t w = q * stride_w + s - pad_w;
                            if (w < 0 || w >= W) continue;
                            const double v = widen(x, x_type, ((n * H + h) * W + w) * C + c);
                            if (inside == 0) acc = v;
                            else if (op == ORACLE_POOL_MAX) acc = v > acc ? v : acc;
                            else if (op == ORACLE_POOL_MIN) acc = v < acc ? v : acc;
                            else acc += v;
                            ++inside;
                        }
                    }
                    if (op == ORACLE_POOL_AVG && inside > 0) acc /= (double)inside;
                    ref[((n * P + p) * Q + q) * C + c] = acc;
                }
    return 0;
}

/* Depthwise 2-D convolution, NHWC: every channel is convolved with its own R x S filter (a grouped
 * convolution with as many groups as channels and one output channel per group). */
int oracle_depthwise_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                                 int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                 const void *input, int in_type, const void *filter, int w_type, int w_layout,
                                 double *ref)
{
    if (N < 0 || H < 0 || W < 0 || C < 0 || R <= 0 || S <= 0) return 1;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return 1;
    if (bad_type(in_type) || bad_type(w_type)) return 2;
    if (w_layout != ORACLE_KRSC && w_layout != ORACLE_RSCK) return 3;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return 0;
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N == 0 || C == 0) return 0;
    if (!input || !filter || !ref) return 4;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t c = 0; c < C; ++c) {
                    double acc = 0.0;
                    for (int64_t r = 0; r < R; ++r) {
                        const int64_t h = p * stride_h + r - pad_h;
                        if (h < 0 || h >= H) continue;
                        for (int64_t s = 0; s < S; ++s) {
                            const int64_t w = q * stride_w + s - pad_w;
                            if (w < 0 || w >= W) continue;
                            const int64_t wi = w_layout == ORACLE_KRSC ? (c * R + r) * S + s : (r * S + s) * C + c;
                            acc += widen(input, in_type, ((n * H + h) * W + w) * C + c) * widen(filter, w_type, wi);
                        }
                    }
                    ref[((n * P + p) * Q + q) * C + c] = acc;
                }
    return 0;
}

/* Convolution with NCHW activations and a KCRS filter: the same sum as oracle_conv2d_nhwc, other strides. */
int oracle_conv2d_nchw(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                       int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                       const void *input, int in_type, const void *filter, int w_type, double *ref)
{
    if (N < 0 || H < 0 || W < 0 || Cin < 0 || Cout < 0 || R <= 0 || S <= 0) return 1;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return 1;
    if (bad_type(in_type) || bad_type(w_type)) return 2;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return 0;
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N == 0 || Cout == 0) return 0;
    if (!ref || (Cin > 0 && (!input || !filter))) return 4;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < Cout; ++k)
            for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < Cin; ++c)
                        for (int64_t r = 0; r < R; ++r) {
                            const int64_t h = p * stride_h + r - pad_h;
                            if (h < 0 || h >= H) continue;
                            for (int64_t s = 0; s < S; ++s) {
                                const int64_t w = q * stride_w + s - pad_w;
                                if (w < 0 || w >= W) continue;
                                acc += widen(input, in_type, ((n * Cin + c) * H + h) * W + w)
                                     * widen(filter, w_type, ((k * Cin + c) * R + r) * S + s);
                            }
                        }
                    ref[((n * Cout + k) * P + p) * Q + q] = acc;
                }
    return 0;
}

/* Multi-scale deformable attention: every query samples each feature level at `points` fractional
 * positions, bilinearly, and adds the samples up with its attention weights. */
int oracle_deformable_attention(int64_t batch, int64_t Lq, int64_t heads, int64_t d, int64_t levels, int64_t points,
                                const void *value, int v_type, const int64_t *level_h, const int64_t *level_w,
                                const float *locations, const float *weights, double *ref)
{
    if (batch < 0 || Lq < 0 || heads < 0 || d < 0 || levels < 0 || points < 0) return 1;
    if (bad_type(v_type)) return 2;
    if (batch == 0 || Lq == 0 || heads == 0 || d == 0) return 0;
    if (!ref || (levels > 0 && (!level_h || !level_w))) return 4;
    int64_t S = 0;
    for (int64_t l = 0; l < levels; ++l) {
        if (level_h[l] < 0 || level_w[l] < 0) return 1;
        S += level_h[l] * level_w[l];
    }
    if (levels > 0 && points > 0 && (!locations || !weights || (S > 0 && !value))) return 4;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < batch; ++n)
        for (int64_t q = 0; q < Lq; ++q)
            for (int64_t m = 0; m < heads; ++m)
                for (int64_t c = 0; c < d; ++c) {
                    double acc = 0.0;
                    int64_t start = 0;                                  /* first row of this level in `value` */
                    for (int64_t l = 0; l < levels; ++l) {
                        const int64_t H = level_h[l], W = level_w[l];
                        for (int64_t p = 0; p < points; ++p) {
                            const int64_t at = (((n * Lq + q) * heads + m) * levels + l) * points + p;
                            /* normalised (x, y) in [0, 1] -> pixel coordinates with pixel centres at i + 0.5 */
                            const double x = (double)locations[2 * at] * (double)W - 0.5;
                            const double y = (double)locations[2 * at + 1] * (double)H - 0.5;
                            /* a full pixel or more outside (or NaN): all four neighbours are padding; also keeps
                             * the conversions to integers below inside their range */
                            if (!(x > -1.0 && x < (double)W && y > -1.0 && y < (double)H)) continue;
                            const double x0 = floor(x), y0 = floor(y);
                            double sample = 0.0;
                            for (int dy = 0; dy < 2; ++dy)
                                for (int dx = 0; dx < 2; ++dx) {
                                    const int64_t xi = (int64_t)x0 + dx, yi = (int64_t)y0 + dy;
                                    if (xi < 0 || xi >= W || yi < 0 || yi >= H) continue;   /* outside: contributes zero */
                                    const double wx = dx ? x - x0 : 1.0 - (x - x0), wy = dy ? y - y0 : 1.0 - (y - y0);
                                    sample += wx * wy * widen(value, v_type, ((n * S + start + yi * W + xi) * heads + m) * d + c);
                                }
                            acc += (double)weights[at] * sample;
                        }
                        start += H * W;
                    }
                    ref[((n * Lq + q) * heads + m) * d + c] = acc;
                }
    return 0;
}
