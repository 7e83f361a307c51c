// What the matrix cores sustain when nothing else happens: a loop of independent MFMAs on operands that
// never leave the registers (no LDS, no memory traffic in the loop).  The throughput of the GEMM kernels
// (the reward of the paper's intra-pass search, Section 5.1, Eq. 3-4) is reported against the chip's
// nominal peak; this kernel gives the second yardstick, the rate the hardware actually holds on random
// operands under its power limit.
//
// One workgroup per compute unit (launched with a dynamic LDS allocation of more than half a compute unit's LDS,
// which keeps a second one away), `waves` waves per
// SIMD, each with the accumulator footprint of a 256 x 256 GEMM tile: 8 x 4 blocks of 16 x 16 (or 4 x 2 of
// 32 x 32) fed from 8 A and 4 B fragments (4 and 2), the same reuse pattern as the GEMM kernels' sub-step.
#include "xp_internal.hpp"

namespace xp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int PAD_LDS = 96 * 1024;                       // more than half of a compute unit's LDS

template <bool INT8, int MF> struct Block;
template <> struct Block<false, 16> {
    typedef f32x4 acc;
    __device__ static acc mma(u32x4 a, u32x4 b, acc c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Block<false, 32> {
    typedef f32x16 acc;
    __device__ static acc mma(u32x4 a, u32x4 b, acc c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Block<true, 16> {
    typedef i32x4 acc;
    __device__ static acc mma(u32x4 a, u32x4 b, acc c)
    {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
    }
};
template <> struct Block<true, 32> {
    typedef i32x16 acc;
    __device__ static acc mma(u32x4 a, u32x4 b, acc c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
    }
};

// operands: per set 12 fragments of 64 lanes x 16 bytes per wave slot (8 wave slots: 96 KB), SETS sets;
// sink: one 32-bit word per thread of the grid.
// 16x16 blocks: two operand sets (the two k sub-steps of a K step), each block takes both back to back on its
// accumulator -- the order that draws the least power of those tried, and the one the GEMM kernel uses.
template <bool INT8, int MF>
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(const u32x4 *operands, unsigned *sink, int iters)
{
    constexpr int MI = MF == 16 ? 8 : 4, NI = MF == 16 ? 4 : 2, NACC = MF == 16 ? 4 : 16, SETS = MF == 16 ? 2 : 1;
    using B = Block<INT8, MF>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    u32x4 a[SETS][MI], b[SETS][NI];
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        const u32x4 *src = operands + ((size_t)(s * 8 + (wave & 7)) * 12) * 64 + lane;
#pragma unroll
        for (int i = 0; i < MI; ++i) a[s][i] = src[i * 64];
#pragma unroll
        for (int j = 0; j < NI; ++j) b[s][j] = src[(8 + j) * 64];
    }
    typename B::acc acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < NACC; ++v) acc[i][j][v] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int jj = 0; jj < NI; ++jj) {
                const int j = (i & 1) ? NI - 1 - jj : jj;
#pragma unroll
                for (int s = 0; s < SETS; ++s) acc[i][j] = B::mma(b[s][j], a[s][i], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
            }
    }
    unsigned x = 0;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < NACC; ++v) {
                if constexpr (INT8) x ^= (unsigned)acc[i][j][v];
                else x ^= __float_as_uint(acc[i][j][v]);
            }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = x;
}

}  // namespace
}  // namespace xp

using namespace xp;

extern "C" {

double xp_mfma_ceiling_ops(xp_dtype in_type, int block, int waves, int64_t iters)
{
    if ((in_type != XP_BF16 && in_type != XP_I8) || (block != 16 && block != 32) || (waves != 1 && waves != 2) || iters < 0) return 0.0;
    const double per_mfma = 2.0 * block * block * (block == 16 ? 32 : 16) * (in_type == XP_I8 ? 2 : 1);
    return 256.0 * 4 * waves * (double)iters * (block == 16 ? 64.0 : 8.0) * per_mfma;
}

xp_status xp_mfma_ceiling(xp_dtype in_type, int block, int waves, int64_t iters, const void *operands, size_t operand_bytes,
                          void *sink, size_t sink_bytes, void *stream)
{
    if ((in_type != XP_BF16 && in_type != XP_I8) || (block != 16 && block != 32) || (waves != 1 && waves != 2)) return XP_ERR_UNSUPPORTED;
    if (iters < 0 || iters > 0x7fffffffLL) return XP_ERR_SHAPE;
    if (!operands || !sink) return XP_ERR_NULL;
    if (((uintptr_t)operands % 16) != 0 || ((uintptr_t)sink % 4) != 0) return XP_ERR_ALIGN;
    const unsigned threads = 256u * (unsigned)waves;
    if (operand_bytes < (size_t)(block == 16 ? 2 : 1) * 8 * 12 * 64 * 16 || sink_bytes < (size_t)256 * threads * 4) return XP_ERR_WORKSPACE;
    const dim3 grid(256), wg(threads);
    hipStream_t s = (hipStream_t)stream;
    const u32x4 *ops = (const u32x4 *)operands;
    unsigned *out = (unsigned *)sink;
    const int n = (int)iters;
    auto launch = [&](auto kernel) {
        // more than 64 KB of dynamic LDS has to be allowed per kernel (a host-side attribute; no device work)
        if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, PAD_LDS) != hipSuccess) return false;
        hipLaunchKernelGGL(kernel, grid, wg, PAD_LDS, s, ops, out, n);
        return true;
    };
    bool ok;
    if (in_type == XP_BF16 && block == 16) ok = launch(mfma_ceiling_kernel<false, 16>);
    else if (in_type == XP_BF16) ok = launch(mfma_ceiling_kernel<false, 32>);
    else if (block == 16) ok = launch(mfma_ceiling_kernel<true, 16>);
    else ok = launch(mfma_ceiling_kernel<true, 32>);
    if (!ok) return XP_ERR_LAUNCH;
    return hipGetLastError() == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

}  // extern "C"
