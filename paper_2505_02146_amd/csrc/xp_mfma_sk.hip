// Single-K-step streaming MFMA kernel: GEMM and strided-batched GEMM whose whole K extent fits one
// 128-byte LDS row (K <= 64 bf16, K <= 128 int8), both operands contiguous along K -- the
// Q.K^T-like first stage of an attention block (Table 5 of the paper: Batch GEMM).  Such a call is
// bound by writing C to HBM, not by the MFMA pipe: what matters is that stores are issued
// continuously and never waited for.
//
// One workgroup owns 64 rows of C and walks all N in tiles of BN columns:
//   * the 64 x K slab of A is read once and kept as MFMA fragments in registers;
//   * a producer wave streams the B tiles into a ring of three LDS buffers with direct
//     global -> LDS loads, two tiles ahead.  Its memory counter sees loads only, so waiting for a
//     tile never waits for a store;
//   * four consumer waves (2 x 2 over the 64 x BN tile) read B fragments, run the MFMAs and store
//     their 32 x BN/2 block of C; stores are fire-and-forget;
//   * one workgroup barrier per tile hands a filled buffer to the consumers and a drained one
//     back to the producer.
// Rows of B past N (and whole tiles past the last one) lie outside the buffer range: the hardware
// writes zeros into LDS and touches no memory, so the producer loop needs no conditionals.
#include "xp_internal.hpp"
#include "xp_epilogue.hpp"

#include <type_traits>

namespace xp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int RB = 128;                   // bytes per LDS row = the whole K extent
constexpr int BM = 64;
constexpr unsigned OOB = 0x80000000u;

struct SkParams {
    const char *A, *B;
    char *C;
    int M, N, Kb;
    long long lda_b, ldb_b, ldc;
    long long strideA_b, strideB_b, strideC;
    float alpha, beta;
    int tiles_n;
};

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// workgroup barrier that the compiler may not move memory accesses across
__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// s_waitcnt immediate for "vmcnt <= n" with lgkmcnt and expcnt left open (gfx9 encoding)
constexpr int waitcnt_vm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }

template <bool INT8> struct Acc;
template <> struct Acc<false> {
    typedef f32x16 type;
    __device__ static __forceinline__ type mma(u32x4 a, u32x4 b, type c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                       c, 0, 0, 0);
    }
};
template <> struct Acc<true> {
    typedef i32x16 type;
    __device__ static __forceinline__ type mma(u32x4 a, u32x4 b, type c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b),
                                                     c, 0, 0, 0);
    }
};

template <bool INT8, int BN, bool STREAM>
__global__ __launch_bounds__(320) void sk_kernel(SkParams p)
{
    using AccT = typename Acc<INT8>::type;
    using OutT = typename std::conditional<INT8, int, float>::type;
    constexpr int NI = BN / 64;                        // 32-column blocks per consumer wave
    constexpr int A_BYTES = BM * RB, B_BYTES = BN * RB;
    constexpr int IB = BN / 8;                         // wave-level loads per B tile (8 rows each)
    static_assert(BN % 64 == 0 && IB <= 31, "tile width");
    __shared__ __attribute__((aligned(1024))) char lds[A_BYTES + 3 * B_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned bx, by;
    xcd_batch_remap(bx, by);                          // the row tiles of one problem share an L2: B is fetched once
    const int m0 = bx * BM;
    const long long batch = by;

    if (wave == 4) {
        // ------------------------------------------------------------------ producer wave
        const __amdgpu_buffer_rsrc_t ra =
            make_rsrc(p.A + batch * p.strideA_b + (long long)m0 * p.lda_b,
                      (unsigned)((long long)(min(p.M - m0, BM) - 1) * p.lda_b + p.Kb));
        const __amdgpu_buffer_rsrc_t rb =
            make_rsrc(p.B + batch * p.strideB_b, (unsigned)((long long)(p.N - 1) * p.ldb_b + p.Kb));
        // lane l of a load lands at row l/8, position l%8 of an 8-row block and fetches the chunk
        // whose swizzled position that is
        const int r8 = lane >> 3;
        auto chunk_of = [&](int row) { return ((lane & 7) ^ swz(row)) << 4; };
#pragma unroll
        for (int i = 0; i < BM / 8; ++i) {
            const int row = i * 8 + r8, cb = chunk_of(row);
            const unsigned off = cb >= p.Kb ? OOB : (unsigned)(row * p.lda_b) + cb;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void *)(lds + i * 1024), 16, off, 0, 0, 0);
        }
        auto issue_b = [&](int j, int buf) {
#pragma unroll
            for (int i = 0; i < IB; ++i) {
                const int row = i * 8 + r8, cb = chunk_of(row);   // BN is a multiple of 16: same swizzle as j*BN + row
                const unsigned off = cb >= p.Kb ? OOB : (unsigned)((j * BN + row) * p.ldb_b) + cb;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void *)(lds + A_BYTES + buf * B_BYTES + i * 1024), 16,
                                                         off, 0, 0, 0);
            }
        };
        issue_b(0, 0);
        issue_b(1, 1);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(IB));     // A and B tile 0 have landed
        wg_barrier();
        int fill = 2;
        for (int j = 0; j < p.tiles_n; ++j) {
            issue_b(j + 2, fill);                       // the buffer the consumers drained in step j-1
            fill = fill == 2 ? 0 : fill + 1;
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(IB)); // B tile j+1 has landed
            wg_barrier();
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        return;
    }

    // ---------------------------------------------------------------------- consumer waves
    const int wm = wave >> 1, wn = wave & 1;
    const int frow = lane & 31, fhi = lane >> 5, fsw = swz(frow);
    int foff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) foff[kk] = frow * RB + (((2 * kk + fhi) ^ fsw) << 4);

    wg_barrier();
    u32x4 af[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) af[kk] = *(const u32x4 *)(lds + wm * 32 * RB + foff[kk]);

    OutT *C = (OutT *)p.C + batch * p.strideC;
    int buf = 0;
    for (int j = 0; j < p.tiles_n; ++j) {
        const char *bt = lds + A_BYTES + buf * B_BYTES + wn * (BN / 2) * RB;
        buf = buf == 2 ? 0 : buf + 1;
        u32x4 bf[NI][4];
#pragma unroll
        for (int b = 0; b < NI; ++b)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) bf[b][kk] = *(const u32x4 *)(bt + b * 32 * RB + foff[kk]);
        AccT acc[NI];
#pragma unroll
        for (int b = 0; b < NI; ++b) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc[b] = Acc<INT8>::mma(af[kk], bf[b][kk], acc[b]);
        }
        // the fragments are in registers (wait for the LDS reads): hand the buffer back before the
        // (long) store phase
        __builtin_amdgcn_s_waitcnt(0xc07f);
        wg_barrier();
#pragma unroll
        for (int b = 0; b < NI; ++b)
            store_block32<INT8, STREAM>(acc[b], C, p.ldc, m0 + wm * 32, j * BN + wn * (BN / 2) + b * 32, lane, p.M, p.N, p.alpha,
                                p.beta);
    }
}

// ------------------------------------------------------------------------------------ host side

template <bool INT8, int BN>
bool sk_can_run(const Problem &q)
{
    if (q.c_plane) return false;                          // planar output: the general and direct-to-LDS kernels only
    const int64_t esz = INT8 ? 1 : 2;
    if (q.in_type != (INT8 ? XP_I8 : XP_BF16) || q.conv) return false;
    if (q.K <= 0 || q.K * esz > RB || (q.K * esz) % 16 != 0) return false;
    if (q.M > 0x7fffffffLL || q.N > 0x3fffffffLL || q.batch > 65535) return false;
    if (q.a_sk != 1 || q.b_sk != 1) return false;
    if ((q.a_sm * esz) % 16 != 0 || (q.b_sn * esz) % 16 != 0) return false;
    if (((uintptr_t)q.A % 16) != 0 || ((uintptr_t)q.B % 16) != 0) return false;
    if ((q.strideA * esz) % 16 != 0 || (q.strideB * esz) % 16 != 0) return false;
    if (BM * q.a_sm * esz >= 0x7fffffffLL) return false;
    if ((q.N + 3 * BN) * q.b_sn * esz >= 0x7fffffffLL) return false;      // row offsets of B, tiles ahead included
    return (q.M + BM - 1) / BM <= 0x7fffffffLL;
}

template <bool INT8, int BN, bool STREAM>
hipError_t sk_launch(const Problem &q)
{
    const int64_t esz = INT8 ? 1 : 2;
    SkParams p;
    p.A = (const char *)q.A; p.B = (const char *)q.B; p.C = (char *)q.C;
    p.M = (int)q.M; p.N = (int)q.N; p.Kb = (int)(q.K * esz);
    p.lda_b = q.a_sm * esz; p.ldb_b = q.b_sn * esz; p.ldc = q.ldc;
    p.strideA_b = q.strideA * esz; p.strideB_b = q.strideB * esz; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    p.tiles_n = (int)((q.N + BN - 1) / BN);
    hipLaunchKernelGGL((sk_kernel<INT8, BN, STREAM>), dim3((unsigned)((q.M + BM - 1) / BM), (unsigned)q.batch), dim3(320), 0,
                       q.stream, p);
    return hipGetLastError();
}

template <int BN>
double sk_cost(const Problem &q)
{
    // bound by writing C: one pass over the output at about 5 TB/s, plus a fixed start-up
    const double wgs = (double)((q.M + BM - 1) / BM) * (double)q.batch;
    const double bytes = (double)q.M * (double)q.N * 4.0 * (double)q.batch;
    const double fill = wgs >= 512.0 ? 1.0 : 512.0 / (wgs + 1.0);
    return 4.0 + fill * bytes / 5e6;
}

#define XP_SK_VARIANT(NAME, TYPESTR, INT8, BN, STREAM, STREAMSTR)                                                      \
    const Variant NAME = {TYPESTR " 64x" #BN "-stream x128B single-k-step producer/consumer" STREAMSTR " mfma32",      \
                          sk_can_run<INT8, BN>, sk_launch<INT8, BN, STREAM>, sk_cost<BN>};

XP_SK_VARIANT(kBfSk64, "bf16", false, 64, false, "")
XP_SK_VARIANT(kBfSk128, "bf16", false, 128, false, "")
XP_SK_VARIANT(kBfSk64nt, "bf16", false, 64, true, " nt-stores")
XP_SK_VARIANT(kBfSk128nt, "bf16", false, 128, true, " nt-stores")
XP_SK_VARIANT(kI8Sk64, "i8", true, 64, false, "")
XP_SK_VARIANT(kI8Sk128, "i8", true, 128, false, "")
XP_SK_VARIANT(kI8Sk128nt, "i8", true, 128, true, " nt-stores")

}  // namespace

int sk_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) { out[0] = &kBfSk64; out[1] = &kBfSk128; out[2] = &kBfSk64nt; out[3] = &kBfSk128nt; return 4; }
    if (in_type == XP_I8) { out[0] = &kI8Sk64; out[1] = &kI8Sk128; out[2] = &kI8Sk128nt; return 3; }
    return 0;
}

}  // namespace xp
