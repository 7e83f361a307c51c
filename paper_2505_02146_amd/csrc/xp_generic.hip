// General kernel: any layout, stride, alignment and size, for GEMM, batched GEMM and the
// im2col view of the NHWC convolution (Table 5 of the paper: GEMM, Batch GEMM, Conv2D NHWC).
// It is the safety net behind the tuned MFMA kernels: LDS-tiled, scalar loads with full
// predication, one fp32 FMA (or int32 multiply-add) per product.  Correct everywhere, fast nowhere.
#include "xp_internal.hpp"

#include <type_traits>

namespace xp {
namespace {

struct GParams {
    const void *A, *B;
    void *C;
    int64_t M, N, K;
    int64_t a_sm, a_sk, b_sk, b_sn, ldc, c_plane;
    int64_t strideA, strideB, strideC;
    float alpha, beta;
    int conv;
    int64_t H, W, Cin, S, P, Q, sh, sw, ph, pw;
};

__device__ inline float widen(float x) { return x; }
__device__ inline float widen(unsigned short x) { return __uint_as_float((unsigned)x << 16); }
__device__ inline int widen(signed char x) { return (int)x; }

constexpr int GT = 64;   // output tile edge
constexpr int GK = 16;   // K step

template <typename TIn, typename TAcc, typename TOut>
__global__ __launch_bounds__(256) void generic_kernel(GParams p)
{
    __shared__ TAcc As[GK][GT + 1];
    __shared__ TAcc Bs[GK][GT + 1];

    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;
    const int64_t m0 = (int64_t)blockIdx.x * GT, n0 = (int64_t)blockIdx.y * GT;
    const int64_t b = blockIdx.z;
    const TIn *A = (const TIn *)p.A + b * p.strideA;
    const TIn *B = (const TIn *)p.B + b * p.strideB;
    TOut *C = (TOut *)p.C + b * p.strideC;

    TAcc acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0;

    // which index runs fastest over the threads of a load: the one that is contiguous in memory
    const bool a_kfast = p.conv || p.a_sk == 1;
    const bool b_kfast = p.b_sk == 1;

    for (int64_t k0 = 0; k0 < p.K; k0 += GK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = t + 256 * i;
            {
                const int r = a_kfast ? e / GK : e % GT;
                const int kk = a_kfast ? e % GK : e / GT;
                const int64_t m = m0 + r, k = k0 + kk;
                TAcc v = 0;
                if (m < p.M && k < p.K) {
                    if (!p.conv) {
                        v = widen(A[m * p.a_sm + k * p.a_sk]);
                    } else {
                        // row m = (n, p, q); column k = (r, s, c)
                        const int64_t n = m / (p.P * p.Q), pq = m % (p.P * p.Q);
                        const int64_t op = pq / p.Q, oq = pq % p.Q;
                        const int64_t tap = k / p.Cin, c = k % p.Cin;
                        const int64_t fr = tap / p.S, fs = tap % p.S;
                        const int64_t h = op * p.sh + fr - p.ph, w = oq * p.sw + fs - p.pw;
                        if (h >= 0 && h < p.H && w >= 0 && w < p.W)
                            v = widen(A[((n * p.H + h) * p.W + w) * p.Cin + c]);
                    }
                }
                As[kk][r] = v;
            }
            {
                const int c = b_kfast ? e / GK : e % GT;
                const int kk = b_kfast ? e % GK : e / GT;
                const int64_t n = n0 + c, k = k0 + kk;
                TAcc v = 0;
                if (n < p.N && k < p.K) v = widen(B[k * p.b_sk + n * p.b_sn]);
                Bs[kk][c] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            TAcc a[4], bb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bb[j] = Bs[kk][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if constexpr (std::is_floating_point<TAcc>::value)
                        acc[i][j] = __builtin_fmaf(a[i], bb[j], acc[i][j]);
                    else
                        acc[i][j] += a[i] * bb[j];
                }
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty + 16 * i;
        if (m >= p.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + tx + 16 * j;
            if (n >= p.N) continue;
            TOut *dst = p.c_plane ? C + ((m / p.c_plane) * p.N + n) * p.c_plane + m % p.c_plane : C + m * p.ldc + n;
            if constexpr (std::is_floating_point<TAcc>::value) {
                float v = p.alpha * acc[i][j];
                if (p.beta != 0.0f) v = __builtin_fmaf(p.beta, *dst, v);
                *dst = v;
            } else {
                *dst = acc[i][j];
            }
        }
    }
}

template <typename TIn, typename TAcc, typename TOut>
hipError_t launch_generic(const Problem &q)
{
    GParams p;
    p.A = q.A; p.B = q.B; p.C = q.C;
    p.M = q.M; p.N = q.N; p.K = q.K;
    p.a_sm = q.a_sm; p.a_sk = q.a_sk; p.b_sk = q.b_sk; p.b_sn = q.b_sn; p.ldc = q.ldc; p.c_plane = q.c_plane;
    p.strideA = q.strideA; p.strideB = q.strideB; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    p.conv = q.conv ? 1 : 0;
    p.H = q.H; p.W = q.W; p.Cin = q.Cin; p.S = q.S; p.P = q.P; p.Q = q.Q;
    p.sh = q.sh; p.sw = q.sw; p.ph = q.ph; p.pw = q.pw;
    const int64_t gx = (q.M + GT - 1) / GT, gy_total = (q.N + GT - 1) / GT;
    // grid.y and grid.z are limited to 65535: walk N in slabs of column tiles, the batch in chunks
    const int64_t slab = 65535;
    const int64_t esz = sizeof(TIn);
    for (int64_t b0 = 0; b0 < q.batch; b0 += slab) {
        const int64_t nb = q.batch - b0 < slab ? q.batch - b0 : slab;
        for (int64_t y0 = 0; y0 < gy_total; y0 += slab) {
            const int64_t ny = gy_total - y0 < slab ? gy_total - y0 : slab;
            GParams s = p;
            const int64_t col0 = y0 * GT;
            s.N = q.N - col0 < ny * GT ? q.N - col0 : ny * GT;
            s.A = (const char *)p.A + b0 * q.strideA * esz;
            s.B = (const char *)p.B + (b0 * q.strideB + col0 * q.b_sn) * esz;
            s.C = (char *)p.C + (b0 * q.strideC + col0) * (int64_t)sizeof(TOut);
            hipLaunchKernelGGL((generic_kernel<TIn, TAcc, TOut>), dim3((unsigned)gx, (unsigned)ny, (unsigned)nb),
                               dim3(256), 0, q.stream, s);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

bool generic_can_run(const Problem &q)
{
    return (q.M + GT - 1) / GT <= 2147483647LL;
}

// VALU rate is a small fraction of any MFMA variant's: price it so that it is only chosen
// when nothing else can run the call.
double generic_cost(const Problem &q)
{
    return 1e3 + 50.0 * tile_cost_us(q, GT, GT, 8320, 256, 0.01, q.in_type == XP_I8 ? 1 : (q.in_type == XP_BF16 ? 2 : 4));
}

const Variant kGenericF32 = {"general f32 64x64x16 valu", generic_can_run, launch_generic<float, float, float>,
                             generic_cost};
const Variant kGenericBF16 = {"general bf16 64x64x16 valu", generic_can_run,
                              launch_generic<unsigned short, float, float>, generic_cost};
const Variant kGenericI8 = {"general i8 64x64x16 valu", generic_can_run, launch_generic<signed char, int, int>,
                            generic_cost};

}  // namespace

int generic_variants(xp_dtype in_type, const Variant **out)
{
    switch (in_type) {
    case XP_F32: out[0] = &kGenericF32; return 1;
    case XP_BF16: out[0] = &kGenericBF16; return 1;
    case XP_I8: out[0] = &kGenericI8; return 1;
    default: return 0;
    }
}

}  // namespace xp
