// Epilogue shared by the MFMA kernels: C = alpha * acc + beta * C for one 32x32 accumulator block.
//
// Accumulator register v of lane l in a 32x32 MFMA block holds row (v/4)*8 + (l>>5)*4 + (v&3),
// column l&31, so one store instruction writes two 128-byte row segments.  Blocks that lie
// completely inside the matrix (the common case) take a branch-free path; beta == 0 never reads C.
#pragma once

#include <hip/hip_runtime.h>

namespace xp {

template <bool INT8, typename AccT, typename OutT>
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
            for (int v = 0; v < 16; ++v) base[(long long)((v >> 2) * 8 + (v & 3)) * ldc] = acc[v];
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
                for (int v = 0; v < 16; ++v) base[(long long)((v >> 2) * 8 + (v & 3)) * ldc] = alpha * acc[v];
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

}  // namespace xp
