/*
 * xp -- dense tensor operators for AMD MI355X (gfx950 / CDNA4), C ABI.
 *
 * The operators are the MatMul and Convolution rows of the benchmark of the QiMeng-Xpiler
 * paper (arXiv 2505.02146, Table 5): GEMM, Batch GEMM and Conv2D NHWC, plus the fused
 * Self Attention operator of its LLM rows.  The paper lists them
 * by name and prints no definition; the standard definitions below are what the library
 * computes.  Every entry point launches hand-written HIP kernels (LDS-tiled, matrix-core
 * MFMA contraction, the kind of instruction Table 1 of the paper names for AMD hardware) on
 * the caller's stream and returns without synchronising.
 *
 * Conventions common to all entry points
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never allocates,
 *     frees or keeps a pointer; there is no hidden workspace.
 *   - Inputs are read-only and may alias each other; the output must not overlap an input.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *     on it; the call does not wait for the GPU.  A stream under HIP graph capture is fine: the
 *     compute entry points enqueue kernels only (the xp_tune_* calls synchronise and are not
 *     capturable).
 *   - Arguments are validated on the host before anything is launched; on error nothing is
 *     launched and a status code is returned.  The library never aborts, throws or prints.
 *   - Supported (A, B -> C) element types: (F32, F32 -> F32), (BF16, BF16 -> F32),
 *     (I8, I8 -> I32).  bf16 is the upper 16 bits of an IEEE fp32; products are accumulated
 *     in fp32 (int32 for I8; signed x signed, two's complement, no saturation).
 *     For I8, alpha must be 1 and beta 0.  Any other combination: XP_ERR_UNSUPPORTED.
 *   - Degenerate sizes: M, N or batch == 0 -> XP_OK, nothing launched.
 *     K == 0 -> C = beta * C (zero-filled when beta == 0).
 *   - beta == 0 means C is not read: NaN or Inf already in C never reach the result.
 *   - Matrices whose layout, alignment or size the tuned kernels do not cover (operands not
 *     contiguous along K, pointers or leading dimensions not multiples of 16 bytes, extents
 *     beyond 32-bit byte offsets within a tile) run on a slower general kernel instead of
 *     failing; the result obeys the same definition.
 *   - Thread safety: entry points may be called concurrently; xp_force_config changes
 *     process-wide state and is meant for tuning sweeps and tests only.
 */
#ifndef XP_H
#define XP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XP_OK = 0,
    XP_ERR_NULL = 1,         /* NULL pointer for a non-empty operand */
    XP_ERR_SHAPE = 2,        /* negative extent, zero filter or stride extent */
    XP_ERR_STRIDE = 3,       /* leading dimension or batch stride smaller than the layout needs */
    XP_ERR_ALIGN = 4,        /* pointer not aligned to its element size */
    XP_ERR_UNSUPPORTED = 5,  /* dtype / layout / alpha-beta combination not provided */
    XP_ERR_CONFIG = 6,       /* forced kernel configuration does not exist or cannot run this call */
    XP_ERR_LAUNCH = 7,       /* the HIP runtime refused the launch */
    XP_ERR_WORKSPACE = 8     /* tuning workspace missing, not 256-byte aligned or too small; file not readable / writable */
} xp_status;

typedef enum { XP_F32 = 0, XP_BF16 = 1, XP_I8 = 2, XP_I32 = 3 } xp_dtype;

/* Layout of a logical matrix X with `rows` x `cols`:
 *   XP_ROW: X(i,j) = X[i*ld + j], ld >= cols;   XP_COL: X(i,j) = X[i + j*ld], ld >= rows. */
typedef enum { XP_ROW = 0, XP_COL = 1 } xp_layout;

/* Filter storage: w(k,r,s,c) for output channel k, tap (r,s), input channel c.
 *   XP_FILTER_KRSC: w[((k*R + r)*S + s)*Cin + c];  XP_FILTER_RSCK: w[((r*S + s)*Cin + c)*Cout + k] */
typedef enum { XP_FILTER_KRSC = 0, XP_FILTER_RSCK = 1 } xp_filter_layout;

/* Operator families for the tuning surface. */
typedef enum { XP_OP_GEMM = 0, XP_OP_GEMM_BATCHED = 1, XP_OP_CONV2D = 2, XP_OP_ATTENTION = 3 } xp_op;

/*
 * GEMM (Table 5, "GEMM"):  C(i,j) = alpha * sum_{k<K} A(i,k) * B(k,j) + beta * C(i,j)
 * for i < M, j < N.  A is the logical M x K matrix, B is K x N, C is M x N, each with its own
 * layout and leading dimension (in elements).  Device pointers; C is written in place.
 */
xp_status xp_gemm(int64_t M, int64_t N, int64_t K, float alpha,
                  const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda,
                  const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb,
                  float beta,
                  void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc,
                  void *stream);

/*
 * Strided-batched GEMM (Table 5, "Batch GEMM"): for every b < batch the GEMM above on
 * A + b*strideA, B + b*strideB, C + b*strideC (strides in elements, >= 0).  strideA or strideB
 * may be 0 to share an operand across the batch; the C slices must not overlap.
 */
xp_status xp_gemm_batched(int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                          const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda, int64_t strideA,
                          const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb, int64_t strideB,
                          float beta,
                          void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc, int64_t strideC,
                          void *stream);

/*
 * 2-D convolution, NHWC (Table 5, "Conv2D NHWC"), computed as an implicit GEMM (the im2col
 * matrix is addressed, never stored):
 *   out[n,p,q,k] = sum_{r<R, s<S, c<Cin} in[n, p*stride_h + r - pad_h, q*stride_w + s - pad_w, c] * w(k,r,s,c)
 * with terms outside the image equal to zero; cross-correlation (no filter flip), dilation 1,
 * one group, no bias.  P = floor((H + 2*pad_h - R)/stride_h) + 1, Q likewise; if the padded image
 * is smaller than the filter the output is empty and XP_OK is returned.
 * input is N x H x W x Cin contiguous, output N x P x Q x Cout contiguous (device pointers).
 * Supported types: (F32, F32 -> F32) and (BF16, BF16 -> F32).
 */
xp_status xp_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                         int64_t R, int64_t S, int64_t stride_h, int64_t stride_w,
                         int64_t pad_h, int64_t pad_w,
                         const void *input, xp_dtype in_type,
                         const void *filter, xp_dtype w_type, xp_filter_layout w_layout,
                         void *output, xp_dtype out_type,
                         void *stream);

/*
 * Fused scaled dot-product attention without a mask (Table 5, "Self Attention"; the paper names
 * the operator and prints no definition, the standard one is computed): for every b < batch,
 *   s(i,j) = scale * sum_{c<d} Q(i,c) K(j,c)            i < Lq, j < Lk
 *   p(i,j) = exp(s(i,j)) / sum_{j'<Lk} exp(s(i,j'))
 *   O(i,x) = sum_{j<Lk} p(i,j) V(j,x)                   x < dv
 * i.e. the two Batch GEMM stages with a row softmax between them, as one kernel that never
 * writes the Lq x Lk score matrix to memory.
 *   Q  batch x Lq x d,  K  batch x Lk x d,  V  batch x Lk x dv,  O  batch x Lq x dv (written).
 * Each is row-major: element (b, i, c) at  base[b*stride + i*ld + c], with the row pitch ld
 * (>= the row length) and the batch stride in elements (>= 0; 0 shares Q, K or V across the
 * batch; the O slices must not overlap).  All four are DEVICE pointers owned by the caller.
 * Supported types: Q, K, V all F32 or all BF16; O is F32.  Products and sums are formed in
 * fp32; on the matrix-core path (BF16, d == dv == 64 or 128, 16-byte aligned pointers, pitches and
 * strides) the probabilities are rounded to bf16 before they multiply V.  Other shapes and
 * alignments run on a slower general kernel under the same definition.
 * scale must be finite (the usual choice is 1/sqrt(d)).
 * Degenerate sizes: batch, Lq or dv == 0 -> XP_OK, nothing launched; d == 0 -> every score is
 * 0, O is the mean of the value rows; Lk == 0 with a non-empty output -> XP_ERR_SHAPE (a
 * softmax over no keys is undefined).
 */
xp_status xp_attention(int64_t batch, int64_t Lq, int64_t Lk, int64_t d, int64_t dv, float scale,
                       const void *Q, xp_dtype q_type, int64_t ldq, int64_t strideQ,
                       const void *K, xp_dtype k_type, int64_t ldk, int64_t strideK,
                       const void *V, xp_dtype v_type, int64_t ldv, int64_t strideV,
                       void *O, xp_dtype o_type, int64_t ldo, int64_t strideO,
                       void *stream);

/*
 * Tuning surface: the stand-in for the tile-size / loop-order / binding knobs that the paper's
 * intra-pass auto-tuning (Section 5.1) searches by brute force.  Every compiled kernel variant
 * of an operator family and input type has an index; a sweep forces each in turn, checks the
 * result and times it, and the winners are recorded in the library's selection table.
 *
 *   xp_num_configs      number of variants for (op, in_type); 0 if none.
 *   xp_describe_config  writes a NUL-terminated description ("bf16 256x256x64 w2x4 st2 ...")
 *                       into buf (at most n bytes).  XP_ERR_CONFIG for a bad index.
 *   xp_force_config     idx >= 0: every later call of that (op, in_type) uses variant idx, and
 *                       returns XP_ERR_CONFIG if the variant cannot run the call's shape or
 *                       layout.  idx < 0: back to the selection table (the default).
 *   xp_last_config      index of the variant the most recent call of (op, in_type) used,
 *                       -1 if none yet.
 */
int xp_num_configs(xp_op op, xp_dtype in_type);
xp_status xp_describe_config(xp_op op, xp_dtype in_type, int idx, char *buf, size_t n);
xp_status xp_force_config(xp_op op, xp_dtype in_type, int idx);
int xp_last_config(xp_op op, xp_dtype in_type);

/*
 * Memory-bound operators (Table 5: Activation -- ReLU, Softmax, GeLU, Sigmoid; Elementwise -- Add,
 * Sign; Pooling -- MaxPool, AvgPool, MinPool, SumPool; LLM -- LayerNorm, RMSNorm; named there without
 * a definition, the standard ones are computed).  Storage types: XP_F32 or XP_BF16 for inputs and,
 * independently, for the output (bf16 output is rounded to nearest even); the arithmetic is fp32.
 * All data pointers are DEVICE pointers; inputs are read-only; in-place use (y == x) is allowed for
 * xp_unary and xp_add with equal input and output types, and for the row-wise operators when, in
 * addition, ldy == ldx.  Empty extents return XP_OK without a launch.
 *
 * Row-wise operators: x is rows x cols, element (i,j) at x[i*ldx + j] (ldx >= cols), y likewise with ldy.
 *   xp_softmax    y(i,j) = exp(x(i,j)) / sum_j' exp(x(i,j'))
 *   xp_layernorm  y(i,j) = (x(i,j) - mean_i) / sqrt(var_i + eps) * gamma(j) + beta(j),
 *                 var_i = (1/cols) sum_j (x(i,j) - mean_i)^2
 *   xp_rmsnorm    y(i,j) = x(i,j) / sqrt((1/cols) sum_j x(i,j)^2 + eps) * gamma(j)
 * gamma and beta are vectors of cols elements of x's type; NULL means all ones / all zeros.
 * eps must be finite and >= 0.  Rows whose length and alignment allow 16-byte accesses (cols a
 * multiple of 4 fp32 / 8 bf16 elements, 16-byte aligned rows) are read from memory exactly once;
 * other rows, and rows longer than 32768 fp32 / 65536 bf16 elements, take a general three-pass kernel.
 */
xp_status xp_softmax(int64_t rows, int64_t cols, const void *x, xp_dtype x_type, int64_t ldx,
                     void *y, xp_dtype y_type, int64_t ldy, void *stream);
xp_status xp_layernorm(int64_t rows, int64_t cols, const void *x, xp_dtype x_type, int64_t ldx,
                       const void *gamma, const void *beta, float eps,
                       void *y, xp_dtype y_type, int64_t ldy, void *stream);
xp_status xp_rmsnorm(int64_t rows, int64_t cols, const void *x, xp_dtype x_type, int64_t ldx,
                     const void *gamma, float eps,
                     void *y, xp_dtype y_type, int64_t ldy, void *stream);

/* Element-wise: relu max(x,0); gelu x/2 (1 + erf(x / sqrt 2)) (the erf form, not the tanh
 * approximation); sigmoid 1 / (1 + exp(-x)); sign -1, 0 or +1; xp_add y = a + b.  n contiguous elements. */
typedef enum { XP_RELU = 0, XP_GELU = 1, XP_SIGMOID = 2, XP_SIGN = 3 } xp_unary_op;
xp_status xp_unary(xp_unary_op op, int64_t n, const void *x, xp_dtype x_type, void *y, xp_dtype y_type, void *stream);
xp_status xp_add(int64_t n, const void *a, const void *b, xp_dtype type, void *y, xp_dtype y_type, void *stream);

/* 2-D pooling, NHWC: x is N x H x W x C contiguous, y is N x P x Q x C contiguous with
 * P = floor((H + 2*pad_h - R)/stride_h) + 1, Q likewise (empty, XP_OK, if the padded image is smaller
 * than the window).  Window positions outside the image do not take part: maximum and minimum are over
 * the positions inside, the sum adds nothing for them, the average divides by the number of
 * positions inside; a window with no position inside gives 0. */
typedef enum { XP_POOL_MAX = 0, XP_POOL_AVG = 1, XP_POOL_MIN = 2, XP_POOL_SUM = 3 } xp_pool_op;
xp_status xp_pool2d_nhwc(xp_pool_op op, int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                         int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                         const void *x, xp_dtype x_type, void *y, xp_dtype y_type, void *stream);

/*
 * 2-D convolution, NCHW (Table 5, "Conv2D NCHW"): the sum of xp_conv2d_nhwc with
 *   input N x Cin x H x W, filter Cout x Cin x R x S (KCRS), output N x Cout x P x Q, all contiguous.
 * It is computed by a change of layout: activations and filter are transposed to NHWC / KRSC in the
 * workspace, the NHWC kernels run and write the N x Cout x P x Q result directly (two extra memory
 * passes over the inputs; callers that can keep their tensors in NHWC should call xp_conv2d_nhwc).
 *   workspace   DEVICE memory owned by the caller, 256-byte aligned, at least
 *               xp_conv2d_nchw_workspace_bytes(...) bytes (0 is returned for invalid or empty shapes);
 *               contents are scratch.  XP_ERR_WORKSPACE if missing, misaligned or too small.
 * Types as for xp_conv2d_nhwc.  N and Cout up to 65535.
 */
size_t xp_conv2d_nchw_workspace_bytes(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                                      int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, xp_dtype in_type);
xp_status xp_conv2d_nchw(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                         int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                         const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                         void *output, xp_dtype out_type, void *workspace, size_t workspace_bytes, void *stream);

/*
 * xp_conv2d_nchw for callers that cannot allocate device memory or pass a workspace of their own: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * result as xp_conv2d_nchw without the workspace: the layout-change passes use a buffer of
 * xp_conv2d_nchw_static_max_bytes() (64 MiB) that is part of the library's device image, one per GPU,
 * held until the process ends.  The call allocates and frees nothing (its first call on a device looks
 * the buffer's address up, once).  A call that needs more than the buffer
 * (xp_conv2d_nchw_workspace_bytes(...) > xp_conv2d_nchw_static_max_bytes()) returns XP_ERR_SHAPE and
 * launches nothing: use xp_conv2d_nchw.  All calls on one GPU share the buffer: calls that may overlap
 * in time there (different streams, or different threads without ordering) race on it and must be
 * serialised by the caller; calls on one stream are ordered by the stream.  Nothing in the buffer has
 * to survive from call to call: every call overwrites the part it reads.
 */
size_t xp_conv2d_nchw_static_max_bytes(void);
xp_status xp_conv2d_nchw_static(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                                int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                                void *output, xp_dtype out_type, void *stream);

/*
 * Multi-scale deformable attention (Table 5, "Deformable Attention"; Section 6 discusses it as the
 * hardest operator of the benchmark).  The operator of Deformable DETR's attention layers:
 *   out[n,q,m,:] = sum_{l<levels, p<points} weights[n,q,m,l,p] * bilinear(value_l[n,:,:,m,:], locations[n,q,m,l,p,:])
 *   value      DEVICE, batch x S x heads x d contiguous, S = sum_l H_l*W_l; level l is stored row-major
 *              (H_l x W_l pixels) after the levels before it.  F32 or BF16.
 *   level_h/w  HOST arrays of `levels` entries (at most 16 levels, each side at most 2^24): read
 *              during the call, not kept.
 *   locations  DEVICE, float, batch x Lq x heads x levels x points x 2: (x, y) relative to the level,
 *              x along the width; the pixel coordinates are x*W - 0.5 and y*H - 0.5 (pixel centres at
 *              half-integers).  8-byte aligned.
 *   weights    DEVICE, float, batch x Lq x heads x levels x points (the caller has normalised them).
 *   out        DEVICE, batch x Lq x heads x d contiguous, F32 or BF16; overwritten.
 * The bilinear sample takes the four pixels around the position; pixels outside the level count as
 * zero, so a position a full pixel or more outside (or NaN) contributes nothing.  Positions are
 * computed in fp32, accumulation is fp32.  levels == 0 or points == 0 writes zeros.  d a multiple of
 * 4 (F32) or 8 (BF16) with 16-byte aligned value/out takes the vectorised kernel.
 */
xp_status xp_deformable_attention(int64_t batch, int64_t Lq, int64_t heads, int64_t d, int64_t levels, int64_t points,
                                  const void *value, xp_dtype v_type, const int64_t *level_h, const int64_t *level_w,
                                  const float *locations, const float *weights, void *out, xp_dtype out_type,
                                  void *stream);

/* Depthwise 2-D convolution, NHWC (Table 5, "Depthwise Conv"): every channel has its own R x S filter,
 *   y[n,p,q,c] = sum_{r<R, s<S} x[n, p*stride_h + r - pad_h, q*stride_w + s - pad_w, c] * w(c,r,s),
 * zero padding, no bias; P, Q as for xp_conv2d_nhwc.  x is N x H x W x C contiguous, y is N x P x Q x C.
 * Filter layouts: XP_FILTER_RSCK  w(c,r,s) = w[(r*S + s)*C + c]  (channel-minor: the fast, vectorised form),
 *                 XP_FILTER_KRSC  w(c,r,s) = w[(c*R + r)*S + s]  (channel-major).
 * x and w share a type (F32 or BF16); y is F32 or BF16; arithmetic fp32.  Memory-bound: one pass. */
xp_status xp_depthwise_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                                   int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                   const void *x, xp_dtype x_type,
                                   const void *w, xp_dtype w_type, xp_filter_layout w_layout,
                                   void *y, xp_dtype y_type, void *stream);

/*
 * Run-time parameter search: the brute-force intra-pass auto-tuning of the paper (Section 5.1) with
 * its reward (Eq. 3-4), inside the library.  xp_tune_* takes the arguments of the entry point it is
 * named after plus a workspace, and
 *   1. computes the call once with the general kernel into the workspace (the reference);
 *   2. forces every variant that accepts the call in turn, into a second workspace copy of C, and
 *      compares it with the reference on the device: a candidate is valid if every element is
 *      finite and the relative Frobenius distance is <= 1e-5 (bit-exact for int8);
 *   3. times each valid candidate (`reps` back-to-back launches between two events, after two
 *      warm-up launches) and the three fastest twice more, in turn; reward = 1 / best time if
 *      valid, else 0; the largest reward wins;
 *   4. records the winner for the call's shape (operator, type, batch, M, N, K, which operands are
 *      contiguous along K, and for a convolution its geometry), so that every later call of that
 *      shape uses it (ahead of the built-in table), and computes C once more with the winner.
 * The calls synchronise `stream` many times and are meant to be made once per shape, off the
 * critical path.  C must hold valid input when beta != 0; it ends up holding the result.
 *   workspace        DEVICE memory owned by the caller, 256-byte aligned, at least
 *                    xp_tune_workspace_bytes(...) bytes; contents are scratch
 *   reps             timed launches per candidate (>= 1)
 *   best, best_us    if not NULL: index of the winning variant (see xp_describe_config) and its
 *                    time per launch in microseconds (HOST pointers)
 * Errors: those of the underlying entry point; XP_ERR_WORKSPACE; XP_ERR_SHAPE for reps < 1.
 * A call with nothing to compute returns XP_OK and records nothing.
 */
xp_status xp_tune_gemm(int64_t M, int64_t N, int64_t K, float alpha,
                       const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda,
                       const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb,
                       float beta,
                       void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc,
                       void *workspace, size_t workspace_bytes, int reps, int *best, float *best_us,
                       void *stream);
xp_status xp_tune_gemm_batched(int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                               const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda, int64_t strideA,
                               const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb, int64_t strideB,
                               float beta,
                               void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc, int64_t strideC,
                               void *workspace, size_t workspace_bytes, int reps, int *best, float *best_us,
                               void *stream);
xp_status xp_tune_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                              int64_t R, int64_t S, int64_t stride_h, int64_t stride_w,
                              int64_t pad_h, int64_t pad_w,
                              const void *input, xp_dtype in_type,
                              const void *filter, xp_dtype w_type, xp_filter_layout w_layout,
                              void *output, xp_dtype out_type,
                              void *workspace, size_t workspace_bytes, int reps, int *best, float *best_us,
                              void *stream);

/* Workspace size for tuning a call whose output spans `c_extent` elements, i.e. from the first to
 * the last element of C including pitch padding and batch gaps:
 * (batch-1)*strideC + (rows-1)*ldc + cols for the stored orientation; N*P*Q*Cout for a convolution. */
size_t xp_tune_workspace_bytes(int64_t c_extent);

/* The table of tuned shapes.  xp_tune_save writes it as text (one shape per line, the variant by
 * name, so that a file survives changes of the variant numbering); xp_tune_load merges a file into
 * the table (later entries replace earlier ones; lines naming unknown variants are kept but have no
 * effect until such a variant exists); xp_tune_clear empties it; xp_tune_count returns its size.
 * Paths are HOST strings.  Thread-safe. */
xp_status xp_tune_save(const char *path);
xp_status xp_tune_load(const char *path);
void xp_tune_clear(void);
int xp_tune_count(void);

/*
 * Measurement aid: the rate the matrix cores sustain on this device when nothing else happens.  The
 * throughput that the paper's parameter search maximises (Section 5.1, Eq. 3-4) is reported against the
 * chip's nominal MFMA peak; this call provides the measured ceiling beside it.  It launches one kernel:
 * one workgroup on each of the 256 compute units, `waves` (1 or 2) waves per SIMD, each running `iters`
 * rounds of 64 16x16 MFMAs (block == 16: 32 blocks, each taking two operand sets back to back on its accumulator,
 * the order that draws the least power; block == 32: 8 independent 32x32 MFMAs) of `in_type`
 * (XP_BF16 or XP_I8) on operands held in registers.  Time it with events on `stream`;
 * xp_mfma_ceiling_ops(...) is the number of arithmetic operations of one launch (0 for invalid arguments).
 *   operands   DEVICE, 16-byte aligned, at least 196608 bytes (block == 32: 98304) of valid `in_type` values (read once, before the loop;
 *              their values set the power drawn: use the distribution of the workload)
 *   sink       DEVICE, at least 256 * 256 * waves * 4 bytes, overwritten (keeps the arithmetic alive)
 * Errors: XP_ERR_UNSUPPORTED (type, block, waves), XP_ERR_SHAPE (iters < 0 or >= 2^31), XP_ERR_NULL, XP_ERR_ALIGN,
 * XP_ERR_WORKSPACE (a buffer too small), XP_ERR_LAUNCH.
 */
double xp_mfma_ceiling_ops(xp_dtype in_type, int block, int waves, int64_t iters);
xp_status xp_mfma_ceiling(xp_dtype in_type, int block, int waves, int64_t iters, const void *operands, size_t operand_bytes,
                          void *sink, size_t sink_bytes, void *stream);

/* Human-readable name of a status code (static storage). */
const char *xp_status_string(xp_status s);

/* Library version string (static storage). */
const char *xp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* XP_H */
