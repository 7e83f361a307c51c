/*
 * Self-test of the CPU oracle, meant to be built with -fsanitize=address,undefined: every operand buffer
 * is heap-allocated at exactly the size the call needs (padded pitches included), so a read or write
 * outside an operand, a signed overflow or a misaligned access stops the program.  The values are
 * checked against closed forms (identity, all-ones sums, int8 extremes, a delta filter, a single key).
 * Test infrastructure like the oracle itself: nothing here is used by the GPU library.
 *
 *   gcc -std=c11 -O1 -g -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan \
 *       -o selftest selftest.c xp_oracle.c -lm && ./selftest
 */
#include "xp_oracle.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static int failures = 0;
#define CHECK(cond, ...)                                                   \
    do {                                                                   \
        if (!(cond)) { ++failures; printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } \
    } while (0)

static uint16_t bf16_of(float x)              /* exact for the small integers used here */
{
    uint32_t u;
    memcpy(&u, &x, 4);
    return (uint16_t)(u >> 16);
}

static float small_int(uint64_t i) { return (float)((int)((i * 2654435761u >> 7) % 17) - 8); }

/* A (M x K) times the identity, in all four layout combinations with padded pitches, both float types */
static void gemm_identity(int type)
{
    const int64_t M = 7, K = 5, pad = 3;
    const size_t esz = type == ORACLE_F32 ? 4 : 2;
    for (int la = 0; la < 2; ++la)
        for (int lb = 0; lb < 2; ++lb) {
            const int64_t lda = (la == ORACLE_ROW ? K : M) + pad, ldb = K + pad;
            const int64_t a_outer = la == ORACLE_ROW ? M : K;
            /* exactly the extent of the layout: the last row or column carries no padding */
            const size_t a_elems = (size_t)((a_outer - 1) * lda + (la == ORACLE_ROW ? K : M));
            const size_t b_elems = (size_t)((K - 1) * ldb + K);
            char *A = malloc(a_elems * esz), *B = malloc(b_elems * esz);
            double *ref = malloc((size_t)(M * K) * sizeof(double));
            memset(A, 0x7f, a_elems * esz);
            memset(B, 0, b_elems * esz);
            for (int64_t i = 0; i < M; ++i)
                for (int64_t k = 0; k < K; ++k) {
                    const size_t at = (size_t)(la == ORACLE_ROW ? i * lda + k : i + k * lda);
                    const float v = small_int((uint64_t)(i * K + k));
                    if (type == ORACLE_F32) ((float *)A)[at] = v;
                    else ((uint16_t *)A)[at] = bf16_of(v);
                }
            for (int64_t k = 0; k < K; ++k) {
                const size_t at = (size_t)(k * ldb + k);
                if (type == ORACLE_F32) ((float *)B)[at] = 1.0f;
                else ((uint16_t *)B)[at] = bf16_of(1.0f);
            }
            const int rc = oracle_gemm_float(M, K, K, 1.0, A, type, la, lda, B, type, lb, ldb, 0.0, NULL, ORACLE_ROW, K, ref);
            CHECK(rc == 0, "gemm identity rc %d", rc);
            for (int64_t i = 0; i < M; ++i)
                for (int64_t k = 0; k < K; ++k)
                    CHECK(ref[i * K + k] == (double)small_int((uint64_t)(i * K + k)), "A.I type %d layouts %d %d at (%d,%d)", type, la, lb, (int)i, (int)k);
            free(A); free(B); free(ref);
        }
}

/* alpha, beta with a padded C0; beta == 0 must not read C0 at all (NULL) */
static void gemm_alpha_beta(void)
{
    const int64_t M = 3, N = 4, K = 6, ldc = N + 2;
    float *A = malloc((size_t)(M * K) * 4), *B = malloc((size_t)(K * N) * 4), *C0 = malloc((size_t)((M - 1) * ldc + N) * 4);
    double *ref = malloc((size_t)(M * N) * 8);
    for (int64_t i = 0; i < M * K; ++i) A[i] = 1.0f;
    for (int64_t i = 0; i < K * N; ++i) B[i] = 1.0f;
    for (int64_t i = 0; i < (M - 1) * ldc + N; ++i) C0[i] = 2.0f;
    CHECK(oracle_gemm_float(M, N, K, 2.0, A, ORACLE_F32, ORACLE_ROW, K, B, ORACLE_F32, ORACLE_ROW, N, 3.0, C0, ORACLE_ROW, ldc, ref) == 0, "rc");
    for (int64_t i = 0; i < M * N; ++i) CHECK(ref[i] == 2.0 * K + 6.0, "alpha beta element %d = %g", (int)i, ref[i]);
    CHECK(oracle_gemm_float(M, N, K, 1.0, A, ORACLE_F32, ORACLE_ROW, K, B, ORACLE_F32, ORACLE_ROW, N, 0.0, NULL, ORACLE_ROW, N, ref) == 0, "rc");
    for (int64_t i = 0; i < M * N; ++i) CHECK(ref[i] == (double)K, "all-ones element %d = %g", (int)i, ref[i]);
    free(A); free(B); free(C0); free(ref);
}

static void gemm_i8_extremes(void)
{
    const int64_t M = 2, N = 3, K = 8192;
    int8_t *A = malloc((size_t)(M * K)), *B = malloc((size_t)(N * K));
    int32_t *ref = malloc((size_t)(M * N) * 4);
    memset(A, 0x80, (size_t)(M * K));                 /* -128 */
    memset(B, 0x80, (size_t)(N * K));
    CHECK(oracle_gemm_i8(M, N, K, A, ORACLE_ROW, K, B, ORACLE_COL, K, ref) == 0, "rc");
    for (int i = 0; i < M * N; ++i) CHECK(ref[i] == 134217728, "(-128)^2 * 8192 = %d", ref[i]);
    memset(B, 0x7f, (size_t)(N * K));                 /* +127: signed x signed */
    CHECK(oracle_gemm_i8(M, N, K, A, ORACLE_ROW, K, B, ORACLE_COL, K, ref) == 0, "rc");
    for (int i = 0; i < M * N; ++i) CHECK(ref[i] == -133169152, "-128 * 127 * 8192 = %d", ref[i]);
    free(A); free(B); free(ref);
}

static void batched_with_gaps(void)
{
    const int64_t b = 3, M = 2, N = 2, K = 3, sA = M * K + 5, sB = K * N + 1;
    float *A = malloc((size_t)((b - 1) * sA + M * K) * 4), *B = malloc((size_t)((b - 1) * sB + K * N) * 4);
    double *ref = malloc((size_t)(b * M * N) * 8);
    for (int64_t i = 0; i < (b - 1) * sA + M * K; ++i) A[i] = 100.0f;    /* gaps hold a value that must not show */
    for (int64_t i = 0; i < (b - 1) * sB + K * N; ++i) B[i] = 100.0f;
    for (int64_t x = 0; x < b; ++x) {
        for (int64_t i = 0; i < M * K; ++i) A[x * sA + i] = (float)(x + 1);
        for (int64_t i = 0; i < K * N; ++i) B[x * sB + i] = 1.0f;
    }
    CHECK(oracle_gemm_float_batched(b, M, N, K, 1.0, A, ORACLE_F32, ORACLE_ROW, K, sA, B, ORACLE_F32, ORACLE_ROW, N, sB, 0.0, NULL,
                                    ORACLE_ROW, N, M * N, ref) == 0, "rc");
    for (int64_t x = 0; x < b; ++x)
        for (int64_t i = 0; i < M * N; ++i) CHECK(ref[x * M * N + i] == (double)((x + 1) * K), "batch %d element %d = %g", (int)x, (int)i, ref[x * M * N + i]);
    free(A); free(B); free(ref);
}

/* delta filter reproduces the image; all-ones counts the taps inside; both filter layouts; stride and padding */
static void conv_closed_forms(void)
{
    const int64_t N = 2, H = 5, W = 4, C = 3;
    const size_t in_elems = (size_t)(N * H * W * C), w_elems = (size_t)(C * 9 * C);
    uint16_t *x = malloc(in_elems * 2), *w = malloc(w_elems * 2);
    double *ref = malloc(in_elems * 8);
    for (size_t i = 0; i < in_elems; ++i) x[i] = bf16_of(small_int(i));
    for (int layout = 0; layout < 2; ++layout) {
        memset(w, 0, w_elems * 2);
        for (int64_t k = 0; k < C; ++k) {
            const int64_t r = 1, s = 1, c = k;
            const size_t at = (size_t)(layout == ORACLE_KRSC ? ((k * 3 + r) * 3 + s) * C + c : ((r * 3 + s) * C + c) * C + k);
            w[at] = bf16_of(1.0f);
        }
        CHECK(oracle_conv2d_nhwc(N, H, W, C, C, 3, 3, 1, 1, 1, 1, x, ORACLE_BF16, w, ORACLE_BF16, layout, ref) == 0, "rc");
        for (size_t i = 0; i < in_elems; ++i) CHECK(ref[i] == (double)small_int(i), "delta filter, layout %d, element %d", layout, (int)i);
    }
    for (size_t i = 0; i < in_elems; ++i) x[i] = bf16_of(1.0f);
    for (size_t i = 0; i < w_elems; ++i) w[i] = bf16_of(1.0f);
    CHECK(oracle_conv2d_nhwc(N, H, W, C, C, 3, 3, 1, 1, 1, 1, x, ORACLE_BF16, w, ORACLE_BF16, ORACLE_KRSC, ref) == 0, "rc");
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < H; ++p)
            for (int64_t q = 0; q < W; ++q) {
                const int rows = 3 - (p == 0) - (p == H - 1), cols = 3 - (q == 0) - (q == W - 1);
                for (int64_t k = 0; k < C; ++k)
                    CHECK(ref[((n * H + p) * W + q) * C + k] == (double)(rows * cols * C), "tap count at (%d,%d)", (int)p, (int)q);
            }
    /* stride 2, no padding: P = 2, Q = 1; output = 9 * C everywhere */
    double *ref2 = malloc((size_t)(N * 2 * 1 * C) * 8);
    CHECK(oracle_conv2d_nhwc(N, H, W, C, C, 3, 3, 2, 2, 0, 0, x, ORACLE_BF16, w, ORACLE_BF16, ORACLE_KRSC, ref2) == 0, "rc");
    for (int64_t i = 0; i < N * 2 * C; ++i) CHECK(ref2[i] == 9.0 * C, "stride 2 element %d = %g", (int)i, ref2[i]);
    free(x); free(w); free(ref); free(ref2);
}

/* one key: the output is that key's value row, whatever the scores; padded pitches */
static void attention_single_key(void)
{
    const int64_t b = 2, Lq = 3, d = 4, dv = 5, ldq = d + 1, ldv = dv + 2;
    float *Q = malloc((size_t)((b - 1) * Lq * ldq + (Lq - 1) * ldq + d) * 4), *K = malloc((size_t)(b * d) * 4);
    float *V = malloc((size_t)((b - 1) * ldv + dv) * 4);
    double *ref = malloc((size_t)(b * Lq * dv) * 8);
    for (int64_t i = 0; i < (b - 1) * Lq * ldq + (Lq - 1) * ldq + d; ++i) Q[i] = small_int((uint64_t)i);
    for (int64_t i = 0; i < b * d; ++i) K[i] = small_int((uint64_t)(i + 77));
    for (int64_t i = 0; i < (b - 1) * ldv + dv; ++i) V[i] = (float)i;
    CHECK(oracle_attention(b, Lq, 1, d, dv, 0.5, Q, ORACLE_F32, ldq, Lq * ldq, K, ORACLE_F32, d, d, V, ORACLE_F32, ldv, ldv, ref) == 0, "rc");
    for (int64_t x = 0; x < b; ++x)
        for (int64_t i = 0; i < Lq; ++i)
            for (int64_t c = 0; c < dv; ++c) CHECK(ref[(x * Lq + i) * dv + c] == (double)(x * ldv + c), "single key, batch %d row %d", (int)x, (int)i);
    free(Q); free(K); free(V); free(ref);
}

static void memory_bound_rows(void)
{
    const int64_t rows = 3, cols = 5, ldx = cols + 3;
    const size_t elems = (size_t)((rows - 1) * ldx + cols);
    float *x = malloc(elems * 4);
    double *ref = malloc((size_t)(rows * cols) * 8);
    for (size_t i = 0; i < elems; ++i) x[i] = 2.0f;
    CHECK(oracle_softmax(rows, cols, x, ORACLE_F32, ldx, ref) == 0, "rc");
    for (int64_t i = 0; i < rows * cols; ++i) CHECK(fabs(ref[i] - 0.2) < 1e-15, "softmax of a constant row = %g", ref[i]);
    CHECK(oracle_layernorm(rows, cols, x, ORACLE_F32, ldx, NULL, NULL, 1e-5, ref) == 0, "rc");
    for (int64_t i = 0; i < rows * cols; ++i) CHECK(ref[i] == 0.0, "layernorm of a constant row = %g", ref[i]);
    CHECK(oracle_rmsnorm(rows, cols, x, ORACLE_F32, ldx, NULL, 0.0, ref) == 0, "rc");
    for (int64_t i = 0; i < rows * cols; ++i) CHECK(fabs(ref[i] - 1.0) < 1e-15, "rmsnorm of a constant row = %g", ref[i]);
    free(x); free(ref);
    /* pooling on an all-ones image: the sum counts the positions inside */
    const int64_t N = 1, H = 4, W = 3, C = 2;
    uint16_t *img = malloc((size_t)(N * H * W * C) * 2);
    double *out = malloc((size_t)(N * H * W * C) * 8);
    for (int64_t i = 0; i < N * H * W * C; ++i) img[i] = bf16_of(1.0f);
    CHECK(oracle_pool2d_nhwc(ORACLE_POOL_SUM, N, H, W, C, 3, 3, 1, 1, 1, 1, img, ORACLE_BF16, out) == 0, "rc");
    for (int64_t p = 0; p < H; ++p)
        for (int64_t q = 0; q < W; ++q) {
            const int cnt = (3 - (p == 0) - (p == H - 1)) * (3 - (q == 0) - (q == W - 1));
            for (int64_t c = 0; c < C; ++c) CHECK(out[(p * W + q) * C + c] == (double)cnt, "sum pool at (%d,%d)", (int)p, (int)q);
        }
    free(img); free(out);
}

/* depthwise and NCHW forms on all-ones data */
static void other_convolutions(void)
{
    const int64_t N = 1, H = 3, W = 3, C = 2;
    float *x = malloc((size_t)(N * H * W * C) * 4), *w = malloc((size_t)(C * 9) * 4), *wd = malloc((size_t)(C * C * 9) * 4);
    double *ref = malloc((size_t)(N * H * W * C) * 8);
    for (int64_t i = 0; i < N * H * W * C; ++i) x[i] = 1.0f;
    for (int64_t i = 0; i < C * 9; ++i) w[i] = 1.0f;
    for (int64_t i = 0; i < C * C * 9; ++i) wd[i] = 1.0f;
    for (int layout = 0; layout < 2; ++layout) {
        CHECK(oracle_depthwise_conv2d_nhwc(N, H, W, C, 3, 3, 1, 1, 1, 1, x, ORACLE_F32, w, ORACLE_F32, layout, ref) == 0, "rc");
        CHECK(ref[(1 * W + 1) * C] == 9.0 && ref[0] == 4.0, "depthwise centre %g corner %g", ref[(1 * W + 1) * C], ref[0]);
    }
    CHECK(oracle_conv2d_nchw(N, H, W, C, C, 3, 3, 1, 1, 1, 1, x, ORACLE_F32, wd, ORACLE_F32, ref) == 0, "rc");
    CHECK(ref[1 * W + 1] == 9.0 * C && ref[0] == 4.0 * C, "nchw centre %g corner %g", ref[1 * W + 1], ref[0]);
    free(x); free(w); free(wd); free(ref);
}

int main(void)
{
    gemm_identity(ORACLE_F32);
    gemm_identity(ORACLE_BF16);
    gemm_alpha_beta();
    gemm_i8_extremes();
    batched_with_gaps();
    conv_closed_forms();
    attention_single_key();
    memory_bound_rows();
    other_convolutions();
    printf(failures ? "oracle selftest: %d failures\n" : "oracle selftest: ok\n", failures);
    return failures ? 1 : 0;
}
