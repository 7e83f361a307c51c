// fp32 x fp32 -> fp32 GEMM and strided-batched GEMM on the fp32 matrix-core instruction
// (32x32x2; Table 1 of the paper names its 16x16x4 sibling as the AMD example), true fp32
// multiplicands, any of the four operand layout combinations.
//
// Both operands are staged through LDS K-major (As[k][m], Bs[k][n]) so that an MFMA fragment
// read (one float per lane: 32 consecutive m or n for a fixed k) is a conflict-free row read,
// whichever way the operand lies in memory.  Global loads are scalar, predicated at the edges,
// and run along the operand's contiguous index.
#include "xp_internal.hpp"

namespace xp {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct FParams {
    const float *A, *B;
    float *C;
    int M, N, K;
    long long a_sm, a_sk, b_sk, b_sn, ldc;
    long long strideA, strideB, strideC;
    float alpha, beta;
    int tiles_n;
};

constexpr int FK = 16;   // K step

template <int BM, int BN>
__global__ __launch_bounds__(256) void f32_kernel(FParams p)
{
    constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;
    constexpr int EA = BM * FK / 256, EB = BN * FK / 256;
    __shared__ float As[FK][BM + 4];
    __shared__ float Bs[FK][BN + 4];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = (blockIdx.x / p.tiles_n) * BM, n0 = (blockIdx.x % p.tiles_n) * BN;
    const long long b = blockIdx.y;
    const float *A = p.A + b * p.strideA;
    const float *B = p.B + b * p.strideB;
    float *C = p.C + b * p.strideC;

    const bool a_kfast = p.a_sk == 1, b_kfast = p.b_sk == 1;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    float ra[EA], rb[EB];
    auto load = [&](int k0) {
#pragma unroll
        for (int i = 0; i < EA; ++i) {
            const int e = t + 256 * i;
            const int r = a_kfast ? e / FK : e % BM, kk = a_kfast ? e % FK : e / BM;
            const int m = m0 + r, k = k0 + kk;
            ra[i] = (m < p.M && k < p.K) ? A[m * p.a_sm + k * p.a_sk] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < EB; ++i) {
            const int e = t + 256 * i;
            const int c = b_kfast ? e / FK : e % BN, kk = b_kfast ? e % FK : e / BN;
            const int n = n0 + c, k = k0 + kk;
            rb[i] = (n < p.N && k < p.K) ? B[k * p.b_sk + n * p.b_sn] : 0.0f;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < EA; ++i) {
            const int e = t + 256 * i;
            const int r = a_kfast ? e / FK : e % BM, kk = a_kfast ? e % FK : e / BM;
            As[kk][r] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < EB; ++i) {
            const int e = t + 256 * i;
            const int c = b_kfast ? e / FK : e % BN, kk = b_kfast ? e % FK : e / BN;
            Bs[kk][c] = rb[i];
        }
    };

    load(0);
    for (int k0 = 0; k0 < p.K; k0 += FK) {
        stage();
        __syncthreads();
        if (k0 + FK < p.K) load(k0 + FK);
        // lane l supplies A(row l&31, k = l>>5) and B(k = l>>5, column l&31) of each 32x32x2 step
#pragma unroll
        for (int kk = 0; kk < FK; kk += 2) {
            float af[MI], bf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = As[kk + (lane >> 5)][wm * WTM + i * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[j] = Bs[kk + (lane >> 5)][wn * WTN + j * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator register v of lane l: row (v/4)*8 + (l>>5)*4 + (v&3), column l&31
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int col = n0 + wn * WTN + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * WTM + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (row < p.M && col < p.N) {
                    float *dst = C + (long long)row * p.ldc + col;
                    float r = p.alpha * acc[i][j][v];
                    if (p.beta != 0.0f) r = __builtin_fmaf(p.beta, *dst, r);
                    *dst = r;
                }
            }
        }
}

bool f32_can_run(const Problem &q)
{
    if (q.c_plane) return false;                          // planar output: the general and direct-to-LDS kernels only
    if (q.in_type != XP_F32 || q.conv) return false;
    if (q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.K > 0x7fffffffLL) return false;
    return q.batch <= 65535 && ((q.M + 63) / 64) * ((q.N + 63) / 64) <= 0x7fffffffLL;
}

template <int BM, int BN>
hipError_t f32_launch(const Problem &q)
{
    FParams p;
    p.A = (const float *)q.A; p.B = (const float *)q.B; p.C = (float *)q.C;
    p.M = (int)q.M; p.N = (int)q.N; p.K = (int)q.K;
    p.a_sm = q.a_sm; p.a_sk = q.a_sk; p.b_sk = q.b_sk; p.b_sn = q.b_sn; p.ldc = q.ldc;
    p.strideA = q.strideA; p.strideB = q.strideB; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    const int tiles_m = (int)((q.M + BM - 1) / BM);
    p.tiles_n = (int)((q.N + BN - 1) / BN);
    hipLaunchKernelGGL((f32_kernel<BM, BN>), dim3((unsigned)(tiles_m * p.tiles_n), (unsigned)q.batch), dim3(256), 0,
                       q.stream, p);
    return hipGetLastError();
}

template <int BM, int BN>
double f32_cost(const Problem &q)
{
    // the fp32 MFMA rate is 1/16 of the bf16 one; the larger tile reuses LDS traffic better
    return tile_cost_us(q, BM, BN, (int)sizeof(float) * FK * (BM + BN + 8), 256, (BM == 128 ? 0.5 : 0.3) / 16.0, 4);
}

const Variant kF32_128 = {"f32 128x128x16 waves 2x2 mfma32x32x2", f32_can_run, f32_launch<128, 128>,
                          f32_cost<128, 128>};
const Variant kF32_64 = {"f32 64x64x16 waves 2x2 mfma32x32x2", f32_can_run, f32_launch<64, 64>, f32_cost<64, 64>};

}  // namespace

int f32_mfma_variants(const Variant **out)
{
    out[0] = &kF32_128;
    out[1] = &kF32_64;
    return 2;
}

}  // namespace xp
