// Matrix-vector products (the MatMul group of Table 5 of the paper holds GEMV-shaped cases next to
// GEMM): a GEMM whose canonical form has N == 1 and whose matrix rows are contiguous along K.
// There is nothing to reuse, every element of A is needed exactly once, so the bound is HBM
// bandwidth and the matrix cores would sit idle: one wave streams one row of A with 16-byte loads
// against the vector (which stays in cache), multiplies in the vector ALUs (fp32 FMA; int8 through
// the 4-way dot instruction), reduces across its lanes and writes one element of C.
// A 1 x N result (M == 1) reaches this file as its transpose: the dispatcher swaps the operands.
#include "xp_internal.hpp"

#include <type_traits>

namespace xp {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct VParams {
    const char *A, *X;
    char *C;
    long long M;
    int K;
    long long lda_b;                       // bytes between rows of A
    long long ldc;                         // elements between entries of the result vector
    long long strideA_b, strideX_b, strideC;
    float alpha, beta;
};

template <xp_dtype T> struct Elem;
template <> struct Elem<XP_F32> { typedef float acc_t; typedef float out_t; static constexpr int SIZE = 4; };
template <> struct Elem<XP_BF16> { typedef float acc_t; typedef float out_t; static constexpr int SIZE = 2; };
template <> struct Elem<XP_I8> { typedef int acc_t; typedef int out_t; static constexpr int SIZE = 1; };

// dot product of two 16-byte chunks
template <xp_dtype T> __device__ __forceinline__ typename Elem<T>::acc_t dot16(u32x4 a, u32x4 x, typename Elem<T>::acc_t acc)
{
    if constexpr (T == XP_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_fmaf(__uint_as_float(a[i]), __uint_as_float(x[i]), acc);
    } else if constexpr (T == XP_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc = __builtin_fmaf(__uint_as_float(a[i] << 16), __uint_as_float(x[i] << 16), acc);
            acc = __builtin_fmaf(__uint_as_float(a[i] & 0xffff0000u), __uint_as_float(x[i] & 0xffff0000u), acc);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_sdot4((int)a[i], (int)x[i], acc, false);
    }
    return acc;
}

template <xp_dtype T> __device__ __forceinline__ typename Elem<T>::acc_t widen1(const char *p, long long i)
{
    if constexpr (T == XP_F32) return ((const float *)p)[i];
    else if constexpr (T == XP_BF16) return __uint_as_float((unsigned)((const unsigned short *)p)[i] << 16);
    else return (int)((const signed char *)p)[i];
}

constexpr int ROWS = 4;                    // rows (= waves) per workgroup
constexpr int UNROLL = 4;                  // 16-byte loads of A in flight per lane

template <xp_dtype T>
__global__ __launch_bounds__(ROWS * 64) void gemv_kernel(VParams p)
{
    using acc_t = typename Elem<T>::acc_t;
    using out_t = typename Elem<T>::out_t;
    constexpr int EPC = 16 / Elem<T>::SIZE;                 // elements per 16-byte chunk
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long row = (long long)blockIdx.x * ROWS + wave;
    if (row >= p.M) return;                                 // whole wave; the kernel has no barrier
    const long long b = blockIdx.y;
    const char *a = p.A + b * p.strideA_b + row * p.lda_b;
    const char *x = p.X + b * p.strideX_b;

    const int chunks = p.K / EPC;
    acc_t acc = 0;
    int c = lane;
    for (; c + 64 * (UNROLL - 1) < chunks; c += 64 * UNROLL) {
        u32x4 av[UNROLL], xv[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            av[u] = __builtin_nontemporal_load((const u32x4 *)a + c + 64 * u);     // used once: do not keep it in cache
            xv[u] = *((const u32x4 *)x + c + 64 * u);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc = dot16<T>(av[u], xv[u], acc);
    }
    for (; c < chunks; c += 64) acc = dot16<T>(__builtin_nontemporal_load((const u32x4 *)a + c), *((const u32x4 *)x + c), acc);
    for (int k = chunks * EPC + lane; k < p.K; k += 64) {  // fewer than EPC elements past the last whole chunk
        if constexpr (T == XP_I8) acc += widen1<T>(a, k) * widen1<T>(x, k);
        else acc = __builtin_fmaf(widen1<T>(a, k), widen1<T>(x, k), acc);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) {
        out_t *dst = (out_t *)p.C + b * p.strideC + row * p.ldc;
        if constexpr (T == XP_I8) {
            *dst = acc;
        } else {
            float v = p.alpha * acc;
            if (p.beta != 0.0f) v = __builtin_fmaf(p.beta, *dst, v);
            *dst = v;
        }
    }
}

template <xp_dtype T>
bool gemv_can_run(const Problem &q)
{
    if (q.c_plane) return false;                          // planar output: the general and direct-to-LDS kernels only
    const int64_t esz = Elem<T>::SIZE;
    if (q.in_type != T || q.conv || q.N != 1 || q.K <= 0) return false;
    if (q.a_sk != 1 || q.b_sk != 1) return false;           // rows of A and the vector contiguous along K
    if (q.K > 0x7fffffffLL || q.batch > 65535 || (q.M + ROWS - 1) / ROWS > 0x7fffffffLL) return false;
    if (((uintptr_t)q.A % 16) != 0 || ((uintptr_t)q.B % 16) != 0) return false;
    if ((q.a_sm * esz) % 16 != 0 || (q.strideA * esz) % 16 != 0 || (q.strideB * esz) % 16 != 0) return false;
    return true;
}

template <xp_dtype T>
hipError_t gemv_launch(const Problem &q)
{
    const int64_t esz = Elem<T>::SIZE;
    VParams p;
    p.A = (const char *)q.A; p.X = (const char *)q.B; p.C = (char *)q.C;
    p.M = q.M; p.K = (int)q.K;
    p.lda_b = q.a_sm * esz; p.ldc = q.ldc;
    p.strideA_b = q.strideA * esz; p.strideX_b = q.strideB * esz; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    hipLaunchKernelGGL(gemv_kernel<T>, dim3((unsigned)((q.M + ROWS - 1) / ROWS), (unsigned)q.batch), dim3(ROWS * 64), 0,
                       q.stream, p);
    return hipGetLastError();
}

template <xp_dtype T>
double gemv_cost(const Problem &q)
{
    // the matrix once at HBM speed, plus launch: below what any tiled kernel estimates for N == 1
    return 1.0 + (double)q.batch * (double)q.M * (double)q.K * Elem<T>::SIZE / 8e6;
}

const Variant kGemvF32 = {"f32 gemv one wave per row", gemv_can_run<XP_F32>, gemv_launch<XP_F32>, gemv_cost<XP_F32>};
const Variant kGemvBf16 = {"bf16 gemv one wave per row", gemv_can_run<XP_BF16>, gemv_launch<XP_BF16>, gemv_cost<XP_BF16>};
const Variant kGemvI8 = {"i8 gemv one wave per row dot4", gemv_can_run<XP_I8>, gemv_launch<XP_I8>, gemv_cost<XP_I8>};

}  // namespace

// Registered after every other family so that the older variants keep their indices.
int gemv_variants(xp_dtype in_type, const Variant **out)
{
    out[0] = in_type == XP_F32 ? &kGemvF32 : (in_type == XP_BF16 ? &kGemvBf16 : &kGemvI8);
    return 1;
}

}  // namespace xp
