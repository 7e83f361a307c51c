// fp32 x fp32 -> fp32 GEMM and strided-batched GEMM on the fp32 matrix-core instruction
// (32x32x2; Table 1 of the paper names its 16x16x4 sibling as the AMD example), true fp32
// multiplicands, any of the four operand layout combinations.
//
// Both operands are staged through LDS K-major (As[k][m], Bs[k][n]) so that an MFMA fragment
// read (one float per lane: 32 consecutive m or n for a fixed k) is a conflict-free row read,
// whichever way the operand lies in memory.  Global loads are scalar, predicated at the edges,
// and run along the operand's contiguous index.
#include "xp_internal.hpp"

#include <type_traits>
#include "xp_epilogue.hpp"

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

// ---------------------------------------------------------------------------------------------
// Pipelined variant.  The fp32 matrix instruction is slow (64 cycles for a 32x32x2 step, 1/16 of the
// bf16 rate), so one wave's fragment reads are cheap beside it and what the kernel has to avoid is
// the matrix pipe standing still: around barriers and while a tile is staged.  Here a K step's
// global loads (16-byte, issued a whole step ahead) sit in registers while the current step is
// multiplied, go into the other LDS buffer at the end of it, and one barrier a step flips the
// buffers.  The layouts are template parameters (KA / KB: operand contiguous along K), the
// staging is K-major as above.  Operands need 16-byte alignment and a multiple of 4 along their
// contiguous index; anything else takes the kernel above.
constexpr int PK = 16;                                   // K step of the pipelined kernel

template <int BM, int BN, bool KA, bool KB>
__global__ __launch_bounds__(256, 4) void f32p_kernel(FParams p)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;
    constexpr int CA = BM * PK / 4 / 256, CB = BN * PK / 4 / 256;          // 16-byte chunks per thread and step
    constexpr int PA = BM + 4, PB = BN + 4;
    __shared__ __attribute__((aligned(16))) float As[2][PK][PA];
    __shared__ __attribute__((aligned(16))) float Bs[2][PK][PB];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = (blockIdx.x / p.tiles_n) * BM, n0 = (blockIdx.x % p.tiles_n) * BN;
    const long long b = blockIdx.y;
    const float *A = p.A + b * p.strideA;
    const float *B = p.B + b * p.strideB;
    float *C = p.C + b * p.strideC;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // chunk e of an operand tile: K-contiguous -> row e / 4, k offset 4 * (e % 4); else k = e / (rows/4),
    // rows 4 * (e % (rows/4)) .. +3.  The loads are buffer loads: the lane's byte offset inside the
    // operand is fixed for the whole loop, the K position of the step is a scalar added by the load
    // itself, and a chunk outside the matrix (a row past M or N, a k past K) has an offset beyond the
    // buffer's range, which reads as zeros -- the loop spends no vector instruction on addresses or
    // bounds, and every vector instruction there is time taken from the matrix pipe.
    constexpr unsigned OUTSIDE = 0x80000000u;            // operands are smaller than 2 GiB
    const unsigned a_bytes = (unsigned)(((KA ? (long long)(p.M - 1) * p.a_sm + p.K : (long long)(p.K - 1) * p.a_sk + p.M)) * 4);
    const unsigned b_bytes = (unsigned)(((KB ? (long long)(p.N - 1) * p.b_sn + p.K : (long long)(p.K - 1) * p.b_sk + p.N)) * 4);
    const __amdgpu_buffer_rsrc_t ra_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(A), 0, a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rb_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(B), 0, b_bytes, 0x00020000);
    unsigned offa[CA], offb[CB];
    int ka[CA], kb[CB];                                   // the chunk's first k inside a step
#pragma unroll
    for (int i = 0; i < CA; ++i) {
        const int e = t + 256 * i;
        if constexpr (KA) {
            const int m = m0 + e / (PK / 4);
            ka[i] = 4 * (e % (PK / 4));
            offa[i] = m < p.M ? (unsigned)(((long long)m * p.a_sm + ka[i]) * 4) : OUTSIDE;
        } else {
            const int m = m0 + 4 * (e % (BM / 4));
            ka[i] = e / (BM / 4);
            offa[i] = m < p.M ? (unsigned)(((long long)ka[i] * p.a_sk + m) * 4) : OUTSIDE;
        }
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
        const int e = t + 256 * i;
        if constexpr (KB) {
            const int n = n0 + e / (PK / 4);
            kb[i] = 4 * (e % (PK / 4));
            offb[i] = n < p.N ? (unsigned)(((long long)n * p.b_sn + kb[i]) * 4) : OUTSIDE;
        } else {
            const int n = n0 + 4 * (e % (BN / 4));
            kb[i] = e / (BN / 4);
            offb[i] = n < p.N ? (unsigned)(((long long)kb[i] * p.b_sk + n) * 4) : OUTSIDE;
        }
    }
    const unsigned step_a = (unsigned)((KA ? 1LL : p.a_sk) * 4), step_b = (unsigned)((KB ? 1LL : p.b_sk) * 4);   // bytes per unit of k
    f32x4 ra[CA], rb[CB];
    // FULL: the whole step lies inside K (every step but possibly the last): nothing to check
    auto load = [&](int k0, bool full) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const unsigned off = full || k0 + ka[i] < p.K ? offa[i] : OUTSIDE;
            ra[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(ra_rsrc, off, (unsigned)k0 * step_a, 0));
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const unsigned off = full || k0 + kb[i] < p.K ? offb[i] : OUTSIDE;
            rb[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb_rsrc, off, (unsigned)k0 * step_b, 0));
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int e = t + 256 * i;
            if constexpr (KA) {
#pragma unroll
                for (int c = 0; c < 4; ++c) As[buf][4 * (e % (PK / 4)) + c][e / (PK / 4)] = ra[i][c];
            } else {
                *(f32x4 *)&As[buf][e / (BM / 4)][4 * (e % (BM / 4))] = ra[i];
            }
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int e = t + 256 * i;
            if constexpr (KB) {
#pragma unroll
                for (int c = 0; c < 4; ++c) Bs[buf][4 * (e % (PK / 4)) + c][e / (PK / 4)] = rb[i][c];
            } else {
                *(f32x4 *)&Bs[buf][e / (BN / 4)][4 * (e % (BN / 4))] = rb[i];
            }
        }
    };
    // lane l supplies A(row l&31, k = l>>5) and B(k = l>>5, column l&31) of each 32x32x2 step
    // the fragments of sub-step kk + 2 are read into a second register set before the matrix
    // instructions of sub-step kk are issued, so that no LDS wait stands between them
    auto multiply = [&](int buf, int kk_begin, int kk_end) {
        float af[2][MI], bf[2][NI];
        auto fetch = [&](int set, int kk) {
#pragma unroll
            for (int i = 0; i < MI; ++i) af[set][i] = As[buf][kk + (lane >> 5)][wm * WTM + i * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[set][j] = Bs[buf][kk + (lane >> 5)][wn * WTN + j * 32 + (lane & 31)];
        };
        fetch(0, kk_begin);
#pragma unroll
        for (int kk = kk_begin; kk < kk_end; kk += 2) {
            const int set = ((kk - kk_begin) >> 1) & 1;
            if (kk + 2 < kk_end) fetch(set ^ 1, kk + 2);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[set][i], bf[set][j], acc[i][j], 0, 0, 0);
        }
    };

    load(0, PK <= p.K);
    stage(0);
    __syncthreads();
    // two steps per trip, so that the buffer index is a constant in every LDS address
    auto step = [&](int k0, auto buf_c) {
        constexpr int buf = decltype(buf_c)::value;
        const bool more = k0 + PK < p.K;                  // uniform
        if (more) load(k0 + PK, k0 + 2 * PK <= p.K);
        multiply(buf, 0, PK);
        if (more) stage(buf ^ 1);                         // the buffer every wave finished reading before the last barrier
        __syncthreads();
    };
    // (no step is conditional inside the loop: a branch around one makes the compiler copy the 64
    // accumulator registers where the paths join)
    const int nsteps = (p.K + PK - 1) / PK;
    int k0 = 0;
    for (int pair = 0; pair < nsteps / 2; ++pair, k0 += 2 * PK) {
        step(k0, std::integral_constant<int, 0>{});
        step(k0 + PK, std::integral_constant<int, 1>{});
    }
    if (nsteps & 1) step(k0, std::integral_constant<int, 0>{});

#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
            store_block32<false>(acc[i][j], C, p.ldc, m0 + wm * WTM + i * 32, n0 + wn * WTN + j * 32, lane, p.M, p.N, p.alpha, p.beta);
}

template <bool KA, bool KB>
bool f32p_can_run(const Problem &q)
{
    if (q.c_plane) return false;
    if (q.in_type != XP_F32 || q.conv || q.K <= 0) return false;
    if (q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.K > 0x7fffffffLL || q.batch > 65535) return false;
    if (((q.M + 63) / 64) * ((q.N + 63) / 64) > 0x7fffffffLL) return false;
    if (((uintptr_t)q.A | (uintptr_t)q.B) % 16 != 0 || q.strideA % 4 != 0 || q.strideB % 4 != 0) return false;
    // buffer addressing: byte offsets inside one operand stay below 2^31
    const int64_t a_ext = KA ? (q.M - 1) * q.a_sm + q.K : (q.K - 1) * q.a_sk + q.M;
    const int64_t b_ext = KB ? (q.N - 1) * q.b_sn + q.K : (q.K - 1) * q.b_sk + q.N;
    if (a_ext * 4 >= 0x7fffffffLL || b_ext * 4 >= 0x7fffffffLL) return false;
    if (KA ? (q.a_sk != 1 || q.a_sm % 4 != 0 || q.K % 4 != 0) : (q.a_sm != 1 || q.a_sk % 4 != 0 || q.M % 4 != 0)) return false;
    if (KB ? (q.b_sk != 1 || q.b_sn % 4 != 0 || q.K % 4 != 0) : (q.b_sn != 1 || q.b_sk % 4 != 0 || q.N % 4 != 0)) return false;
    return true;
}

template <int BM, int BN, bool KA, bool KB>
hipError_t f32p_launch(const Problem &q)
{
    FParams p;
    p.A = (const float *)q.A; p.B = (const float *)q.B; p.C = (float *)q.C;
    p.M = (int)q.M; p.N = (int)q.N; p.K = (int)q.K;
    p.a_sm = q.a_sm; p.a_sk = q.a_sk; p.b_sk = q.b_sk; p.b_sn = q.b_sn; p.ldc = q.ldc;
    p.strideA = q.strideA; p.strideB = q.strideB; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    const int tiles_m = (int)((q.M + BM - 1) / BM);
    p.tiles_n = (int)((q.N + BN - 1) / BN);
    hipLaunchKernelGGL((f32p_kernel<BM, BN, KA, KB>), dim3((unsigned)(tiles_m * p.tiles_n), (unsigned)q.batch), dim3(256), 0,
                       q.stream, p);
    return hipGetLastError();
}

template <int BM, int BN>
double f32p_cost(const Problem &q)
{
    return tile_cost_us(q, BM, BN, 2 * (int)sizeof(float) * PK * (BM + BN + 8), 256, (BM == 128 ? 0.8 : 0.5) / 16.0, 4);
}

#define XP_F32P(NAME, BM, BN, KA, KB, LAY)                                                                      \
    const Variant NAME = {"f32 " #BM "x" #BN "x16 waves 2x2 pipelined " LAY " mfma32x32x2", f32p_can_run<KA, KB>, \
                          f32p_launch<BM, BN, KA, KB>, f32p_cost<BM, BN>};
XP_F32P(kF32P128_kk, 128, 128, true, true, "A,B along K")
XP_F32P(kF32P128_km, 128, 128, true, false, "A along K, B along N")
XP_F32P(kF32P128_mk, 128, 128, false, true, "A along M, B along K")
XP_F32P(kF32P128_mm, 128, 128, false, false, "A along M, B along N")
XP_F32P(kF32P64_kk, 64, 64, true, true, "A,B along K")
XP_F32P(kF32P64_km, 64, 64, true, false, "A along K, B along N")
XP_F32P(kF32P64_mk, 64, 64, false, true, "A along M, B along K")
XP_F32P(kF32P64_mm, 64, 64, false, false, "A along M, B along N")
#undef XP_F32P

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

// ---------------------------------------------------------------------------------------------
// Small problems (a few dozen tiles, K of a few hundred): what such a call costs is latency, not throughput.
// The tiled kernels above walk K in steps of 16 with the next step's loads one step ahead -- a quarter of a
// microsecond of MFMA work to cover a load that takes three times as long, sixteen times in a row for K = 256.
// Here a workgroup owns a 32 x 32 tile of C (many workgroups even for a small C), brings a whole chunk of 256 k
// of both operands into LDS with every load of the chunk in flight at once (one memory latency per chunk), and
// its four waves each multiply a quarter of the chunk's k range into their own copy of the tile, which are
// added up through LDS at the end (wave 0 + wave 1 + wave 2 + wave 3, always in that order).
constexpr int SK = 256;                                  // k per chunk
constexpr int ST = 32;                                   // tile edge

// LA, LB: how A and B are brought in. 0: any strides, one element per load. 1: the operand is contiguous along k
// (row-major A, column-major B), 2: contiguous along its own index (column-major A, row-major B); both with every
// extent, pitch and pointer that the 16-byte loads touch a multiple of four elements. A k-contiguous operand stays
// [index][k] in LDS (pitch 260 floats) and a lane reads four consecutive k of its row with one 16-byte read; the
// other form is [k][index] (pitch 36). The lanes of the lower half of a wave take k = 8q .. 8q+3, those of the upper
// half 8q+4 .. 8q+7, for A and B alike, so that the four MFMA steps of a group pair equal k (the order of the sum
// over k is free).
template <int L>
struct F32sOperand {
    static constexpr int E4 = ST * SK / 256 / 4;         // 16-byte groups per thread and chunk
    static constexpr int PITCH = L == 1 ? SK + 4 : ST + 4;
    static constexpr int FLOATS = L == 1 ? ST * PITCH : SK * PITCH;
    typedef float f32x4v __attribute__((ext_vector_type(4)));
    // group e of the chunk: (index, k) of its first element
    static __device__ __forceinline__ void where(int e, int &idx, int &kk)
    {
        if constexpr (L == 1) { idx = e / (SK / 4); kk = 4 * (e % (SK / 4)); }
        else { kk = e / (ST / 4); idx = 4 * (e % (ST / 4)); }
    }
    // pitch: elements between consecutive values of the slow index (rows for L == 1, k for L == 2)
    static __device__ __forceinline__ void load(f32x4v (&r)[E4], const float *P, long long pitch, int i0, int I, int k0, int K, int t)
    {
#pragma unroll
        for (int i = 0; i < E4; ++i) {
            int idx, kk;
            where(t + 256 * i, idx, kk);
            const bool ok = i0 + idx < I && k0 + kk < K;                           // I or K is a multiple of 4: a group is whole or absent
            const long long off = L == 1 ? (long long)(i0 + idx) * pitch + (k0 + kk) : (long long)(k0 + kk) * pitch + (i0 + idx);
            r[i] = ok ? *(const f32x4v *)(P + off) : f32x4v{0.0f, 0.0f, 0.0f, 0.0f};
        }
    }
    static __device__ __forceinline__ void store(float *S, const f32x4v (&r)[E4], int t)
    {
#pragma unroll
        for (int i = 0; i < E4; ++i) {
            int idx, kk;
            where(t + 256 * i, idx, kk);
            *(f32x4v *)&S[L == 1 ? idx * PITCH + kk : kk * PITCH + idx] = r[i];
        }
    }
    // the four values k .. k+3 of this lane's row or column
    static __device__ __forceinline__ f32x4v read(const float *S, int idx, int k)
    {
        if constexpr (L == 1) return *(const f32x4v *)&S[idx * PITCH + k];
        else return f32x4v{S[k * PITCH + idx], S[(k + 1) * PITCH + idx], S[(k + 2) * PITCH + idx], S[(k + 3) * PITCH + idx]};
    }
};

template <int LA, int LB>
__global__ __launch_bounds__(256) void f32s_kernel(FParams p)
{
    static_assert((LA == 0) == (LB == 0), "both operands by 16-byte loads, or neither");
    constexpr bool VEC = LA != 0;
    constexpr int E = ST * SK / 256;                     // elements per thread, operand and chunk
    constexpr int APITCH = ST + 4;                       // the one-element form keeps both operands [k][index]
    typedef F32sOperand<VEC ? LA : 2> OA;
    typedef F32sOperand<VEC ? LB : 2> OB;
    __shared__ __attribute__((aligned(16))) float As[OA::FLOATS];
    __shared__ __attribute__((aligned(16))) float Bs[OB::FLOATS];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int m0 = (blockIdx.x / p.tiles_n) * ST, n0 = (blockIdx.x % p.tiles_n) * ST;
    const long long b = blockIdx.y;
    const float *A = p.A + b * p.strideA;
    const float *B = p.B + b * p.strideB;
    float *C = p.C + b * p.strideC;
    const bool a_kfast = p.a_sk == 1, b_kfast = p.b_sk == 1;

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    for (int k0 = 0; k0 < p.K; k0 += SK) {
        if constexpr (VEC) {
            typename OA::f32x4v ra[OA::E4], rb[OB::E4];
            OA::load(ra, A, LA == 1 ? p.a_sm : p.a_sk, m0, p.M, k0, p.K, t);
            OB::load(rb, B, LB == 1 ? p.b_sn : p.b_sk, n0, p.N, k0, p.K, t);
            if (k0 > 0) __syncthreads();                 // the chunk before has been multiplied by every wave
            OA::store(As, ra, t);
            OB::store(Bs, rb, t);
            __syncthreads();
            const int kq = wave * (SK / 4) + 4 * (lane >> 5);
#pragma unroll
            for (int g = 0; g < SK / 4; g += 8) {
                const auto a4 = OA::read(As, lane & 31, kq + g);
                const auto b4 = OB::read(Bs, lane & 31, kq + g);
#pragma unroll
                for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[u], b4[u], acc, 0, 0, 0);
            }
        } else {
        float ra[E], rb[E];
        // consecutive threads take consecutive elements along the operand's contiguous index
#pragma unroll
        for (int i = 0; i < E; ++i) {
            const int e = t + 256 * i;
            const int r = a_kfast ? e / SK : e % ST, kk = a_kfast ? e % SK : e / ST;
            const int m = m0 + r, k = k0 + kk;
            ra[i] = (m < p.M && k < p.K) ? A[m * p.a_sm + k * p.a_sk] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < E; ++i) {
            const int e = t + 256 * i;
            const int c = b_kfast ? e / SK : e % ST, kk = b_kfast ? e % SK : e / ST;
            const int n = n0 + c, k = k0 + kk;
            rb[i] = (n < p.N && k < p.K) ? B[k * p.b_sk + n * p.b_sn] : 0.0f;
        }
        if (k0 > 0) __syncthreads();                     // the chunk before has been multiplied by every wave
#pragma unroll
        for (int i = 0; i < E; ++i) {
            const int e = t + 256 * i;
            As[(a_kfast ? e % SK : e / ST) * APITCH + (a_kfast ? e / SK : e % ST)] = ra[i];
            Bs[(b_kfast ? e % SK : e / ST) * APITCH + (b_kfast ? e / SK : e % ST)] = rb[i];
        }
        __syncthreads();
        // this wave's quarter of the chunk; lane l supplies A(row l&31, k = l>>5) and B(k = l>>5, column l&31)
        const int kq = wave * (SK / 4);
#pragma unroll 8
        for (int kk = 0; kk < SK / 4; kk += 2) {
            const float af = As[(kq + kk + (lane >> 5)) * APITCH + (lane & 31)], bf = Bs[(kq + kk + (lane >> 5)) * APITCH + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, acc, 0, 0, 0);
        }
        }
    }

    // the four partial tiles through LDS (As is free after the barrier); thread t then owns 4 accumulator
    // registers of one lane position: register v of lane l is row (v/4)*8 + (l>>5)*4 + (v&3), column l&31
    __syncthreads();
    float *red = &As[0];                                 // 4 x 16 x 64 floats = 16 KB of the 33 KB or more
#pragma unroll
    for (int v = 0; v < 16; ++v) red[(wave * 16 + v) * 64 + lane] = acc[v];
    __syncthreads();
    const int col = n0 + (lane & 31);
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int v = wave * 4 + x;
        const float sum = ((red[(0 * 16 + v) * 64 + lane] + red[(1 * 16 + v) * 64 + lane]) + red[(2 * 16 + v) * 64 + lane]) +
                          red[(3 * 16 + v) * 64 + lane];
        const int row = m0 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (row < p.M && col < p.N) {
            float *dst = C + (long long)row * p.ldc + col;
            float r = p.alpha * sum;
            if (p.beta != 0.0f) r = __builtin_fmaf(p.beta, *dst, r);
            *dst = r;
        }
    }
}

bool f32s_can_run(const Problem &q)
{
    if (q.c_plane || q.in_type != XP_F32 || q.conv || q.K <= 0) return false;
    if (q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.K > 0x7fffffffLL || q.batch > 65535) return false;
    return ((q.M + ST - 1) / ST) * ((q.N + ST - 1) / ST) <= 0x7fffffffLL;
}

// 1: 16-byte loads along k, 2: 16-byte loads along the operand's own index, 0: neither is possible
int f32s_form(const Problem &q, bool is_a)
{
    const long long s_idx = is_a ? q.a_sm : q.b_sn, s_k = is_a ? q.a_sk : q.b_sk, ext = is_a ? q.M : q.N;
    const long long stride = is_a ? q.strideA : q.strideB;
    const uintptr_t ptr = (uintptr_t)(is_a ? q.A : q.B);
    if (ptr % 16 != 0 || stride % 4 != 0) return 0;
    if (s_k == 1 && s_idx % 4 == 0 && q.K % 4 == 0) return 1;
    if (s_idx == 1 && s_k % 4 == 0 && ext % 4 == 0) return 2;
    return 0;
}

hipError_t f32s_launch(const Problem &q)
{
    FParams p;
    p.A = (const float *)q.A; p.B = (const float *)q.B; p.C = (float *)q.C;
    p.M = (int)q.M; p.N = (int)q.N; p.K = (int)q.K;
    p.a_sm = q.a_sm; p.a_sk = q.a_sk; p.b_sk = q.b_sk; p.b_sn = q.b_sn; p.ldc = q.ldc;
    p.strideA = q.strideA; p.strideB = q.strideB; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    const int tiles_m = (int)((q.M + ST - 1) / ST);
    p.tiles_n = (int)((q.N + ST - 1) / ST);
    const dim3 grid((unsigned)(tiles_m * p.tiles_n), (unsigned)q.batch);
    const int la = f32s_form(q, true), lb = f32s_form(q, false);
    if (la == 1 && lb == 1) hipLaunchKernelGGL((f32s_kernel<1, 1>), grid, dim3(256), 0, q.stream, p);
    else if (la == 1 && lb == 2) hipLaunchKernelGGL((f32s_kernel<1, 2>), grid, dim3(256), 0, q.stream, p);
    else if (la == 2 && lb == 1) hipLaunchKernelGGL((f32s_kernel<2, 1>), grid, dim3(256), 0, q.stream, p);
    else if (la == 2 && lb == 2) hipLaunchKernelGGL((f32s_kernel<2, 2>), grid, dim3(256), 0, q.stream, p);
    else hipLaunchKernelGGL((f32s_kernel<0, 0>), grid, dim3(256), 0, q.stream, p);
    return hipGetLastError();
}

// Calibrated on the device (calls replayed from a HIP graph). With 16-byte loads: about 2.4 us per launch and 2 us
// per chunk of 256 k (256^3 4.4 us, 512 x 512 x 1024 11.2 us, 64 x 64 x 4096 33 us, each ahead of the tiled kernels:
// 8.4, 26.5, 97). One element per load: 3 us and 4.5 us per chunk. With more than one workgroup per compute unit the
// tiled kernels win (1024^2 x 256: 11.0 against 9.3)
double f32s_cost(const Problem &q)
{
    const double tiles = (double)((q.M + ST - 1) / ST) * (double)((q.N + ST - 1) / ST) * (double)q.batch;
    if (tiles > 256.0 || q.K > 8192) return 1e30;
    const double chunks = (double)((q.K + SK - 1) / SK);
    return f32s_form(q, true) && f32s_form(q, false) ? 2.4 + 2.0 * chunks : 3.0 + 4.5 * chunks;
}

const Variant kF32_small = {"f32 32x32x256 four waves split k, whole chunk in flight, mfma32x32x2", f32s_can_run, f32s_launch, f32s_cost};

const Variant kF32_128 = {"f32 128x128x16 waves 2x2 mfma32x32x2", f32_can_run, f32_launch<128, 128>,
                          f32_cost<128, 128>};
const Variant kF32_64 = {"f32 64x64x16 waves 2x2 mfma32x32x2", f32_can_run, f32_launch<64, 64>, f32_cost<64, 64>};

}  // namespace

int f32_mfma_variants(const Variant **out)
{
    const Variant *all[] = {&kF32_128, &kF32_64, &kF32P128_kk, &kF32P128_km, &kF32P128_mk, &kF32P128_mm,
                            &kF32P64_kk, &kF32P64_km, &kF32P64_mk, &kF32P64_mm};
    for (int i = 0; i < 10; ++i) out[i] = all[i];
    return 10;
}

// Registered after the other fp32 families: their indices stay as they were.
int f32_small_variants(const Variant **out)
{
    out[0] = &kF32_small;
    return 1;
}

}  // namespace xp
