// Internal declarations shared by the host-side dispatcher and the kernel translation units.
// Nothing here is part of the C ABI (that is include/xp.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xp.h"

namespace xp {

// A call after canonicalisation: C is row-major (c_sn == 1), every operand is described by two
// element strides, and a convolution is a GEMM whose A operand is the (virtual) im2col matrix:
//   row m = (n, p, q) of the output, column k = (r, s, c) of the filter window.
struct Problem {
    xp_op op;
    xp_dtype in_type;             // XP_F32, XP_BF16 or XP_I8 (both inputs)
    int64_t batch, M, N, K;
    const void *A, *B;
    void *C;
    int64_t a_sm, a_sk;           // A(i,k) = A[i*a_sm + k*a_sk]   (unused for conv)
    int64_t b_sk, b_sn;           // B(k,j) = B[k*b_sk + j*b_sn]
    int64_t ldc;                  // C(i,j) = C[i*ldc + j]
    int64_t strideA, strideB, strideC;
    float alpha, beta;
    bool conv;
    int64_t H, W, Cin, R, S, P, Q, sh, sw, ph, pw;
    hipStream_t stream;
};

// One compiled kernel variant: a point in the tile / wave-grid / pipeline-depth space.
struct Variant {
    const char *name;
    bool (*can_run)(const Problem &);
    hipError_t (*launch)(const Problem &);
    double (*cost)(const Problem &);   // estimated run time, arbitrary units, lower is better
};

// Variant tables, one per input type.  Index 0 is always the general (any layout) kernel.
int num_variants(xp_dtype in_type);
const Variant *variant(xp_dtype in_type, int idx);

// Registration hooks implemented by the kernel translation units.
int generic_variants(xp_dtype in_type, const Variant **out);
int f32_mfma_variants(const Variant **out);
int kc_variants(xp_dtype in_type, const Variant **out);
int dl_variants(xp_dtype in_type, const Variant **out);
int oc_variants(xp_dtype in_type, const Variant **out);

inline int elem_size(xp_dtype t) { return t == XP_F32 || t == XP_I32 ? 4 : (t == XP_BF16 ? 2 : 1); }

}  // namespace xp
