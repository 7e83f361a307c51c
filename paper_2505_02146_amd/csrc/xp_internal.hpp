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
    int64_t c_plane;              // > 0: planar output instead (NCHW convolution results), C(i,j) =
                                  // C[((i / c_plane) * N + j) * c_plane + i % c_plane]; ldc unused; beta == 0
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

// Fused attention has its own problem description and its own (short) variant table.
struct AttnProblem {
    xp_dtype in_type;             // XP_F32 or XP_BF16 (Q, K and V alike); the output is fp32
    int64_t batch, Lq, Lk, d, dv;
    float scale;
    const void *Q, *K, *V;
    void *O;
    int64_t ldq, ldk, ldv, ldo;   // row pitches, elements
    int64_t strideQ, strideK, strideV, strideO;
    hipStream_t stream;
};
struct AttnVariant {
    const char *name;
    bool (*can_run)(const AttnProblem &);
    hipError_t (*launch)(const AttnProblem &);
    bool (*worthwhile)(const AttnProblem &) = nullptr;   // selection skips a variant that can run but would not pay; null: always
};
int attn_num_variants(xp_dtype in_type);                    // index 0 is the general kernel
const AttnVariant *attn_variant(xp_dtype in_type, int idx);

// Variant tables, one per input type.  Index 0 is always the general (any layout) kernel.
int num_variants(xp_dtype in_type);
const Variant *variant(xp_dtype in_type, int idx);

// Registration hooks implemented by the kernel translation units.
int generic_variants(xp_dtype in_type, const Variant **out);
int f32_mfma_variants(const Variant **out);
int f32_small_variants(const Variant **out);
int kc_variants(xp_dtype in_type, const Variant **out);
int dl_variants(xp_dtype in_type, const Variant **out);
int oc_variants(xp_dtype in_type, const Variant **out);
int sk_variants(xp_dtype in_type, const Variant **out);
int pp_variants(xp_dtype in_type, const Variant **out);
int dl_asym_variants(xp_dtype in_type, const Variant **out);
int dl_bnm_variants(xp_dtype in_type, const Variant **out);
int dl_asm_variants(xp_dtype in_type, const Variant **out);
int dl_small_variants(xp_dtype in_type, const Variant **out);
int rs_variants(xp_dtype in_type, const Variant **out);
int dl_pair_variants(xp_dtype in_type, const Variant **out);
int gemv_variants(xp_dtype in_type, const Variant **out);

// Pieces of the dispatcher that the run-time tuner uses (xp_api.hip).
xp_status make_gemm_problem(xp_op op, int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                            const void *A, xp_dtype a_t, xp_layout a_l, int64_t lda, int64_t strideA,
                            const void *B, xp_dtype b_t, xp_layout b_l, int64_t ldb, int64_t strideB,
                            float beta, void *C, xp_dtype c_t, xp_layout c_l, int64_t ldc, int64_t strideC,
                            void *stream, Problem *out, bool *nothing);
xp_status make_conv_problem(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                            int64_t R, int64_t S, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                            const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                            xp_filter_layout w_layout, void *output, xp_dtype out_type, void *stream,
                            Problem *out, bool *nothing);
xp_status launch_variant(const Problem &q, int idx);      // that variant or XP_ERR_CONFIG; no selection
xp_status run(const Problem &q);                          // forced variant, else selection
// Table of shapes tuned at run time or loaded from a file (xp_tune.hip): index of the recorded
// variant if the shape is known and the variant can run the call, else -1.
void selection_changed();                                   // the run-time table changed: forget remembered selections
int runtime_tuned_variant(const Problem &q);

// Run-time estimate (microseconds) shared by the MFMA variants' cost functions, used only for shapes
// that are not in the table of swept winners.  conc = workgroups that fit one compute unit;
// a round of workgroups takes the largest of MFMA time at the swept efficiency, HBM time for the
// C tile plus L2 time for the operand tiles, and a fixed per-workgroup latency.
inline double tile_cost_us(const Problem &q, int BM, int BN, int lds_bytes, int threads, double eff, int esz)
{
    const double tiles = (double)((q.M + BM - 1) / BM) * (double)((q.N + BN - 1) / BN) * (double)q.batch;
    int conc = lds_bytes > 0 ? (160 * 1024) / lds_bytes : 8;
    if (conc > 2048 / threads) conc = 2048 / threads;
    if (conc > 8) conc = 8;
    if (conc < 1) conc = 1;
    const double slots = 256.0 * conc;
    const double rounds = conc == 1 ? __builtin_ceil(tiles / slots) : (tiles <= slots ? 1.0 : tiles / slots);
    // workgroups that actually share a compute unit: fewer than conc when the grid is small
    double share = tiles >= slots ? (double)conc : __builtin_ceil(tiles / 256.0);
    if (share < 1.0) share = 1.0;
    const double rate = esz == 1 ? 2.0 * 9.83e6 : 9.83e6;             // MFMA flop per microsecond per compute unit
    const double t_comp = 2.0 * BM * BN * (double)q.K / (rate * eff) * share;
    const double t_mem = share * ((double)BM * BN * 4.0 / 16e3 + (double)(BM + BN) * (double)q.K * esz / 64e3);
    const double t_lat = 3.0;
    const double t_work = t_comp > t_mem ? t_comp : t_mem;
    return conc == 1 ? rounds * (t_work + t_lat) : rounds * (t_work > t_lat ? t_work : t_lat);
}

// Batched launches with few tiles per problem: the workgroups of one problem have consecutive
// linear ids and would be dealt round-robin to the 8 XCDs, so each XCD's L2 would fetch that
// problem's operands again.  This renumbering gives XCD x (linear id mod 8) a contiguous run of
// (tile, batch) pairs instead, so a problem's tiles share one L2.  Returns the renumbered
// blockIdx.x in `x` and blockIdx.y in `y`; identity when the grid size is not a multiple of 8.
__device__ __forceinline__ void xcd_batch_remap(unsigned &x, unsigned &y)
{
    const unsigned gx = gridDim.x, total = gx * gridDim.y;
    x = blockIdx.x;
    y = blockIdx.y;
    if ((total & 7) == 0) {
        const unsigned lin = y * gx + x;
        const unsigned ren = (lin & 7) * (total >> 3) + (lin >> 3);
        x = ren % gx;
        y = ren / gx;
    }
}

// One-dimensional launches whose neighbouring workgroups share cache lines (window overlap, the heads
// of a pixel): workgroups are dealt round-robin to the 8 XCDs, so XCD x (linear id mod 8) takes a
// contiguous eighth of the work instead of every eighth item.  The grid must be a multiple of 8;
// ids beyond the number of items come out >= that number and the caller skips them.
__device__ __forceinline__ unsigned xcd_chunked(unsigned linear, unsigned grid)
{
    return (linear & 7u) * (grid >> 3) + (linear >> 3);
}

inline int elem_size(xp_dtype t) { return t == XP_F32 || t == XP_I32 ? 4 : (t == XP_BF16 ? 2 : 1); }

}  // namespace xp
