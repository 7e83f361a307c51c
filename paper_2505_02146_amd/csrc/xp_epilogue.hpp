// Epilogue shared by the MFMA kernels: C = alpha * acc + beta * C for one 32x32 accumulator block.
//
// Accumulator register v of lane l in a 32x32 MFMA block holds row (v/4)*8 + (l>>5)*4 + (v&3),
// column l&31, so one store instruction writes two 128-byte row segments.  Blocks that lie
// completely inside the matrix (the common case) take a branch-free path; beta == 0 never reads C.
#pragma once

#include <hip/hip_runtime.h>

namespace xp {

// STREAM = true marks the stores non-temporal: for outputs that are written once and not read again
// by the kernel (the store-bound batched shapes) they should not displace operand lines in the caches.
template <bool STREAM, typename T> __device__ __forceinline__ void put(T *dst, T v)
{
    if constexpr (STREAM) __builtin_nontemporal_store(v, dst);
    else *dst = v;
}

template <bool INT8, bool STREAM = false, typename AccT, typename OutT>
__device__ __forceinline__ void store_block32(const AccT &acc, OutT *C, long long ldc, int blk_row0, int blk_col0,
                                              int lane, int M, int N, float alpha, float beta)
{
    const int col = blk_col0 + (lane & 31);
    const int row0 = blk_row0 + (lane >> 5) * 4;
    OutT *base = C + (long long)row0 * ldc + col;
    const bool interior = blk_row0 + 32 <= M && blk_col0 + 32 <= N;
    if constexpr (INT8) {
        if (interior) {
#pragma unroll
            for (int v = 0; v < 16; ++v) put<STREAM>(base + (long long)((v >> 2) * 8 + (v & 3)) * ldc, (OutT)acc[v]);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = (v >> 2) * 8 + (v & 3);
                if (row0 + r < M && col < N) base[(long long)r * ldc] = acc[v];
            }
        }
    } else {
        if (beta == 0.0f) {
            if (interior) {
#pragma unroll
                for (int v = 0; v < 16; ++v) put<STREAM>(base + (long long)((v >> 2) * 8 + (v & 3)) * ldc, alpha * acc[v]);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = (v >> 2) * 8 + (v & 3);
                    if (row0 + r < M && col < N) base[(long long)r * ldc] = alpha * acc[v];
                }
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = (v >> 2) * 8 + (v & 3);
                if (row0 + r < M && col < N) {
                    OutT *dst = base + (long long)r * ldc;
                    *dst = __builtin_fmaf(beta, *dst, alpha * acc[v]);
                }
            }
        }
    }
}

// 16x16 block computed transposed (B fragment as the first MFMA operand): accumulator register v
// of lane l holds C(row l&15, column 4*(l>>4) + v), i.e. 4 consecutive columns: one 16-byte store
// per lane when the address is 16-byte aligned and the block is interior.
template <bool INT8, bool STREAM = false, typename AccT, typename OutT>
__device__ __forceinline__ void store_block16t(const AccT &acc, OutT *C, long long ldc, int blk_row0, int blk_col0,
                                               int lane, int M, int N, float alpha, float beta)
{
    const int row = blk_row0 + (lane & 15);
    const int col0 = blk_col0 + (lane >> 4) * 4;
    OutT *dst = C + (long long)row * ldc + col0;
    const bool interior = blk_row0 + 16 <= M && blk_col0 + 16 <= N;
    const bool vec_ok = interior && (((unsigned long long)C | (unsigned long long)(ldc * (long long)sizeof(OutT))) & 15) == 0 &&
                        (blk_col0 & 3) == 0;
    typedef OutT out4 __attribute__((ext_vector_type(4)));
    if constexpr (INT8) {
        if (vec_ok) {
            put<STREAM>((out4 *)dst, out4{acc[0], acc[1], acc[2], acc[3]});
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (row < M && col0 + v < N) dst[v] = acc[v];
        }
    } else {
        if (beta == 0.0f && vec_ok) {
            put<STREAM>((out4 *)dst, out4{alpha * acc[0], alpha * acc[1], alpha * acc[2], alpha * acc[3]});
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (row < M && col0 + v < N) {
                    float r = alpha * acc[v];
                    if (beta != 0.0f) r = __builtin_fmaf(beta, dst[v], r);
                    dst[v] = r;
                }
        }
    }
}

// The same transposed 16x16 block into a planar output: row i (a pixel) of column j (a channel) lives at
// ((i / plane) * N + j) * plane + i % plane.  For each of a lane's four columns the 16 lanes l&15
// write 16 consecutive rows: one 64-byte run of a plane while the rows stay inside one image.
template <typename AccT, typename OutT>
__device__ __forceinline__ void store_block16t_planar(const AccT &acc, OutT *C, long long plane, int blk_row0, int blk_col0,
                                                      int lane, int M, int N, float alpha)
{
    const int row = blk_row0 + (lane & 15);
    const int col0 = blk_col0 + (lane >> 4) * 4;
    if (row >= M) return;
    // (rows and planes are below 2^31 here: a 32-bit division, a quarter of the instructions of a 64-bit one)
    const unsigned img = (unsigned)row / (unsigned)plane, pix = (unsigned)row - img * (unsigned)plane;
    OutT *dst = C + ((long long)img * N + col0) * plane + pix;
#pragma unroll
    for (int v = 0; v < 4; ++v)
        if (col0 + v < N) dst[v * plane] = (OutT)(alpha * acc[v]);
}

}  // namespace xp
