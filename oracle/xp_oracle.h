/*
 * CPU oracle for the dense tensor operators of the MatMul and Convolution groups of the
 * paper's benchmark (Table 5: GEMM, Batch GEMM, Conv2D NHWC) and for the fused attention operator
 * of its LLM group (Table 5: Self Attention), and for the memory-bound operators of its Activation,
 * Elementwise, Pooling and LLM groups.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It exists so that the GPU library can be
 * checked against something that is obviously right.  It is plain, slow, scalar C: the
 * textbook definition of each operator written out, with fp64 accumulation for floating-point
 * inputs and int64 accumulation for int8 inputs.  No blocking, no intrinsics, no BLAS, and no
 * code, header, table or helper shared with the GPU library.  OpenMP is used only to run
 * independent output rows in parallel; the summation order inside one output element is always
 * k ascending (for convolution: r, then s, then c ascending).
 *
 * The paper names the operators (Table 5) but prints no definition of them; the definitions
 * used are the standard ones:
 *   GEMM        ref(i,j) = alpha * sum_k A(i,k) B(k,j) + beta * C0(i,j)      (beta == 0: C0 unread)
 *   batched     the same for every batch index on pointers advanced by the batch strides
 *   conv NHWC   ref[n,p,q,k] = sum_{r,s,c} in[n, p*sh + r - ph, q*sw + s - pw, c] * w(k,r,s,c)
 *               (cross-correlation, zero padding, dilation 1, groups 1, no bias)
 *   attention   ref = softmax_over_keys(scale * Q K^T) V, no mask, for every batch index
 *
 * All pointers are host pointers.  Reference outputs are dense and row-major
 * (M x N, batch x M x N, N x P x Q x Cout) regardless of the layout of the operands.
 * Every function returns 0 on success and a positive code on a bad argument.
 */
#ifndef XP_ORACLE_H
#define XP_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of floating-point operands */
#define ORACLE_F32  0
#define ORACLE_BF16 1   /* uint16 bit pattern, widened exactly */

/* layouts of the logical matrices */
#define ORACLE_ROW 0    /* X(i,j) = X[i*ld + j] */
#define ORACLE_COL 1    /* X(i,j) = X[i + j*ld] */

/* filter layouts */
#define ORACLE_KRSC 0   /* w(k,r,s,c) = w[((k*R + r)*S + s)*Cin + c]  */
#define ORACLE_RSCK 1   /* w(k,r,s,c) = w[((r*S + s)*Cin + c)*Cout + k] */

/* Floating-point GEMM.  A is M x K, B is K x N, C0 (fp32, may be NULL when beta == 0) is M x N.
 * ref receives M*N doubles, row-major. */
int oracle_gemm_float(int64_t M, int64_t N, int64_t K, double alpha,
                      const void *A, int a_type, int a_layout, int64_t lda,
                      const void *B, int b_type, int b_layout, int64_t ldb,
                      double beta, const float *C0, int c_layout, int64_t ldc,
                      double *ref);

/* int8 x int8 -> int32 GEMM with int64 accumulation.  Returns 0, or 100 if any exact sum
 * falls outside the int32 range (ref then holds the truncated value). */
int oracle_gemm_i8(int64_t M, int64_t N, int64_t K,
                   const int8_t *A, int a_layout, int64_t lda,
                   const int8_t *B, int b_layout, int64_t ldb,
                   int32_t *ref);

/* Strided-batched floating-point GEMM: for every b the single GEMM on A + b*strideA etc.
 * (strides in elements).  ref receives batch*M*N doubles. */
int oracle_gemm_float_batched(int64_t batch, int64_t M, int64_t N, int64_t K, double alpha,
                              const void *A, int a_type, int a_layout, int64_t lda, int64_t strideA,
                              const void *B, int b_type, int b_layout, int64_t ldb, int64_t strideB,
                              double beta, const float *C0, int c_layout, int64_t ldc, int64_t strideC,
                              double *ref);

/* Direct convolution, seven nested loops.  input is N x H x W x Cin contiguous, ref receives
 * N*P*Q*Cout doubles with P = (H + 2*pad_h - R)/stride_h + 1 (floor), Q likewise. */
int oracle_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                       int64_t R, int64_t S, int64_t stride_h, int64_t stride_w,
                       int64_t pad_h, int64_t pad_w,
                       const void *input, int in_type,
                       const void *filter, int w_type, int w_layout,
                       double *ref);

/* Scaled dot-product attention without a mask (the "Self Attention" operator of Table 5; the
 * paper prints no definition, the standard one is used):
 *   s(i,j) = scale * sum_c Q(i,c) K(j,c),   p(i,j) = exp(s(i,j)) / sum_j' exp(s(i,j')),
 *   ref(i,x) = sum_j p(i,j) V(j,x)
 * for every batch index.  Q is batch x Lq x d, K is batch x Lk x d, V is batch x Lk x dv; each
 * is row-major with a row pitch (ldq, ldk, ldv) and a batch stride, both in elements.  Lk must
 * be positive.  ref receives batch*Lq*dv doubles, dense.  Everything is computed in fp64. */
int oracle_attention(int64_t batch, int64_t Lq, int64_t Lk, int64_t d, int64_t dv, double scale,
                     const void *Q, int q_type, int64_t ldq, int64_t strideQ,
                     const void *K, int k_type, int64_t ldk, int64_t strideK,
                     const void *V, int v_type, int64_t ldv, int64_t strideV,
                     double *ref);

/* Memory-bound operators of Table 5 (Activation: ReLU, Softmax, GeLU, Sigmoid; Elementwise: Add,
 * Sign; Pooling: MaxPool, AvgPool, MinPool, SumPool; LLM: LayerNorm, RMSNorm), named there without a
 * definition; the standard ones, in fp64:
 *   softmax    y(i,j) = exp(x(i,j)) / sum_j' exp(x(i,j'))                     over the last dimension
 *   layernorm  y(i,j) = (x(i,j) - mean_i) / sqrt(var_i + eps) * gamma(j) + beta(j), var_i = mean of squares of deviations
 *   rmsnorm    y(i,j) = x(i,j) / sqrt(mean_j x(i,j)^2 + eps) * gamma(j)
 *   relu max(x,0); gelu x/2 (1 + erf(x/sqrt 2)); sigmoid 1/(1+exp(-x)); sign -1, 0 or +1; add a + b
 *   pooling    NHWC, window R x S, strides, zero-free padding (positions outside the image do not take part)
 * x is rows x cols with row pitch ldx (elements); ref is dense.  gamma / beta have x's element type, NULL = 1 / 0. */
#define ORACLE_RELU 0
#define ORACLE_GELU 1
#define ORACLE_SIGMOID 2
#define ORACLE_SIGN 3
#define ORACLE_POOL_MAX 0
#define ORACLE_POOL_AVG 1
#define ORACLE_POOL_MIN 2
#define ORACLE_POOL_SUM 3
int oracle_softmax(int64_t rows, int64_t cols, const void *x, int x_type, int64_t ldx, double *ref);
int oracle_layernorm(int64_t rows, int64_t cols, const void *x, int x_type, int64_t ldx,
                     const void *gamma, const void *beta, double eps, double *ref);
int oracle_rmsnorm(int64_t rows, int64_t cols, const void *x, int x_type, int64_t ldx,
                   const void *gamma, double eps, double *ref);
int oracle_unary(int op, int64_t n, const void *x, int x_type, double *ref);
int oracle_add(int64_t n, const void *a, const void *b, int type, double *ref);
int oracle_pool2d_nhwc(int op, int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                       int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                       const void *x, int x_type, double *ref);

/* Depthwise convolution, NHWC (Table 5: Depthwise Conv): out[n,p,q,c] = sum_{r,s} in[n, p*sh + r - ph, q*sw + s - pw, c] * w(c,r,s),
 * zero padding, no bias.  Filter layouts: ORACLE_KRSC  w(c,r,s) = w[(c*R + r)*S + s]  (channel-major),
 * ORACLE_RSCK  w(c,r,s) = w[(r*S + s)*C + c]  (channel-minor). */
int oracle_depthwise_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                                 int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                 const void *input, int in_type, const void *filter, int w_type, int w_layout,
                                 double *ref);

/* Convolution, NCHW (Table 5: Conv2D NCHW): input N x Cin x H x W, filter Cout x Cin x R x S, ref N x Cout x P x Q;
 * out[n,k,p,q] = sum_{c,r,s} in[n, c, p*sh + r - ph, q*sw + s - pw] * w[k,c,r,s], zero padding, no bias. */
int oracle_conv2d_nchw(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                       int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                       const void *input, int in_type, const void *filter, int w_type, double *ref);

/* Multi-scale deformable attention (Table 5: Deformable Attention; the operator of Deformable DETR):
 *   out[n,q,m,:] = sum_{l<levels, p<points} weights[n,q,m,l,p] * bilinear(value_l[n,:,:,m,:], locations[n,q,m,l,p,:])
 * value is batch x S x heads x d with S = sum_l H_l*W_l, level l stored row-major (H_l x W_l) after the
 * levels before it; locations are (x, y) in [0,1] relative to the level (x along the width), mapped to
 * pixel coordinates x*W - 0.5, y*H - 0.5 (pixel centres at half-integers); the bilinear sample takes the
 * four surrounding pixels, those outside the level count as zero.  locations: batch x Lq x heads x
 * levels x points x 2 floats; weights: the same without the last axis; ref: batch x Lq x heads x d. */
int oracle_deformable_attention(int64_t batch, int64_t Lq, int64_t heads, int64_t d, int64_t levels, int64_t points,
                                const void *value, int v_type, const int64_t *level_h, const int64_t *level_w,
                                const float *locations, const float *weights, double *ref);

/* Number of OpenMP threads the loops above will use. */
int oracle_num_threads(void);
/* Caps the threads of those loops (n <= 0: back to the default).  Bookkeeping for timing, no arithmetic. */
void oracle_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
