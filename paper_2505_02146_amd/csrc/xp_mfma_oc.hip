// MFMA kernels for GEMM and strided-batched GEMM whose operands are NOT both contiguous along K
// (bf16 and int8; Table 5 of the paper: GEMM, Batch GEMM): row-major B ("NN", the second stage of
// an attention block), column-major A, or both.
//
// The MFMA instruction wants, per lane, consecutive K elements of one row of A / column of B.  An
// operand that is contiguous along its outer index (m or n) instead is staged in LDS in a
// "K-group interleaved" layout: G = 4/sizeof(element) consecutive k values of one column are
// packed into one 32-bit word (a byte/half-word permute in registers on the way from global
// memory to LDS), and the words of one K group are stored contiguously along the outer index:
//     lds[kg][x]  (32-bit words),  word = { X(k = kg*G .. kg*G+G-1, x) }
// A fragment is then 4 word reads per lane (K groups kk*8 + 4*(lane/32) + 0..3, column lane%32),
// each conflict-free because 32 consecutive lanes read 32 consecutive words.  Operands that are
// contiguous along K use the same swizzled 128-byte-row layout as the other MFMA kernels.
//
// The pipeline is the plain two-buffer one (global loads for step t+1 in registers while step t
// is multiplied, one workgroup barrier per step): the shapes this kernel serves are bound by
// HBM bandwidth or are small, and several workgroups per compute unit hide the latency.
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

constexpr int ROWB = 128;                 // bytes of K per step
constexpr int KG = 32;                    // 4-byte K groups per step
constexpr unsigned OOB = 0x80000000u;

struct OcParams {
    const char *A, *B;
    char *C;
    int M, N, K;                          // elements
    long long lda_b, ldb_b;               // leading dimensions in bytes
    long long ldc;
    long long strideA_b, strideB_b, strideC;
    float alpha, beta;
    int tiles_n;
};

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

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

// One operand tile (ROWS outer elements x one K step) in LDS, its staging registers and its
// fragment reads.  OC = contiguous along the outer index in memory.
template <bool INT8, int ROWS, int NT, bool OC>
struct Operand {
    static constexpr int ESZ = INT8 ? 1 : 2;
    static constexpr int G = 4 / ESZ;                                 // k values per 32-bit word
    static constexpr int XCH = ROWS * ESZ / 16;                       // 16-byte chunks along the outer index
    static constexpr int PITCH = ROWS * 4 + 32;                       // bytes per K-group row (OC layout)
    static constexpr int BYTES = OC ? KG * PITCH : ROWS * ROWB;       // LDS bytes per buffer
    static constexpr int NTASK = OC ? KG * XCH : ROWS * 8;            // staging tasks per step
    static constexpr int PER = (NTASK + NT - 1) / NT;                 // tasks per thread
    static constexpr int NREG = OC ? PER * G : PER;
    static_assert(NTASK % NT == 0 || NTASK < NT, "staging tasks must divide evenly over the workgroup");

    u32x4 g[NREG];

    // KC: range ends after the last valid row; OC: after the last valid k row of this column window
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int tid, int kt, long long ld_b, int Kb)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int q = tid + i * NT;
            if (NTASK < NT && q >= NTASK) continue;
            if constexpr (!OC) {
                const int row = q >> 3, chunk = q & 7;
                const int kb = kt * ROWB;
                unsigned off = (unsigned)(row * ld_b) + (chunk << 4);
                if (kb + (chunk << 4) >= Kb) off = OOB;
                g[i] = __builtin_amdgcn_raw_buffer_load_b128(r, off, kb, 0);
            } else {
                const int xc = q % XCH, kg = q / XCH;
                const int k0 = kt * (ROWB / ESZ) + kg * G;
#pragma unroll
                for (int j = 0; j < G; ++j)
                    g[i * G + j] = __builtin_amdgcn_raw_buffer_load_b128(r, (unsigned)((k0 + j) * ld_b) + (xc << 4), 0, 0);
            }
        }
    }

    __device__ __forceinline__ void store(char *base, int tid) const
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int q = tid + i * NT;
            if (NTASK < NT && q >= NTASK) continue;
            if constexpr (!OC) {
                const int row = q >> 3, chunk = q & 7;
                *(u32x4 *)(base + row * ROWB + ((chunk ^ swz(row)) << 4)) = g[i];
            } else {
                const int xc = q % XCH, kg = q / XCH;
                char *dst = base + kg * PITCH + xc * (16 / ESZ) * 4;
                if constexpr (!INT8) {
                    // rows k, k+1 of 8 columns -> 8 words {X(k,x), X(k+1,x)}
                    const u32x4 r0 = g[i * 2], r1 = g[i * 2 + 1];
                    u32x4 lo, hi;
#pragma unroll
                    for (int d = 0; d < 2; ++d) {
                        lo[2 * d] = (r0[d] & 0xffffu) | (r1[d] << 16);
                        lo[2 * d + 1] = (r0[d] >> 16) | (r1[d] & 0xffff0000u);
                        hi[2 * d] = (r0[d + 2] & 0xffffu) | (r1[d + 2] << 16);
                        hi[2 * d + 1] = (r0[d + 2] >> 16) | (r1[d + 2] & 0xffff0000u);
                    }
                    *(u32x4 *)dst = lo;
                    *(u32x4 *)(dst + 16) = hi;
                } else {
                    // rows k..k+3 of 16 columns -> 16 words of 4 bytes
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        u32x4 w;
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const int sh = 8 * b;
                            w[b] = ((g[i * 4][d] >> sh) & 0xffu) | (((g[i * 4 + 1][d] >> sh) & 0xffu) << 8) |
                                   (((g[i * 4 + 2][d] >> sh) & 0xffu) << 16) | (((g[i * 4 + 3][d] >> sh) & 0xffu) << 24);
                        }
                        *(u32x4 *)(dst + 16 * d) = w;
                    }
                }
            }
        }
    }

    // fragment of the 32-row block starting at outer index x0, MFMA sub-step kk
    __device__ static __forceinline__ u32x4 frag(const char *base, int x0, int kk, int lane)
    {
        const int r = lane & 31, kh = lane >> 5;
        if constexpr (!OC) {
            const int row = x0 + r;
            return *(const u32x4 *)(base + row * ROWB + (((2 * kk + kh) ^ swz(row)) << 4));
        } else {
            u32x4 v;
            const char *src = base + (kk * 8 + kh * 4) * PITCH + (x0 + r) * 4;
#pragma unroll
            for (int d = 0; d < 4; ++d) v[d] = *(const unsigned *)(src + d * PITCH);
            return v;
        }
    }
};

template <bool INT8, int BM, int BN, int WM, int WN, bool A_OC, bool B_OC>
__global__ __launch_bounds__(WM *WN * 64) void oc_kernel(OcParams p)
{
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN, MI = WTM / 32, NI = WTN / 32;
    constexpr int ESZ = INT8 ? 1 : 2;
    using OpA = Operand<INT8, BM, NT, A_OC>;
    using OpB = Operand<INT8, BN, NT, B_OC>;
    using AccT = typename Acc<INT8>::type;
    constexpr int STAGE = OpA::BYTES + OpB::BYTES;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave sub-tile must be whole MFMA blocks");
    static_assert(2 * STAGE <= 160 * 1024, "LDS budget");
    __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    unsigned bx, by;
    xcd_batch_remap(bx, by);                          // the tiles of one problem share an L2
    const int m0 = (bx / p.tiles_n) * BM, n0 = (bx % p.tiles_n) * BN;
    const long long batch = by;
    const int Kb = p.K * ESZ;

    __amdgpu_buffer_rsrc_t ra, rb;
    if constexpr (A_OC)      // A(i,k) at k*lda + i: window of columns m0.., all k rows
        ra = make_rsrc(p.A + batch * p.strideA_b + (long long)m0 * ESZ,
                       (unsigned)((long long)(p.K - 1) * p.lda_b + (long long)(p.M - m0) * ESZ));
    else
        ra = make_rsrc(p.A + batch * p.strideA_b + (long long)m0 * p.lda_b,
                       (unsigned)((long long)(min(p.M - m0, BM) - 1) * p.lda_b + Kb));
    if constexpr (B_OC)      // B(k,j) at k*ldb + j
        rb = make_rsrc(p.B + batch * p.strideB_b + (long long)n0 * ESZ,
                       (unsigned)((long long)(p.K - 1) * p.ldb_b + (long long)(p.N - n0) * ESZ));
    else
        rb = make_rsrc(p.B + batch * p.strideB_b + (long long)n0 * p.ldb_b,
                       (unsigned)((long long)(min(p.N - n0, BN) - 1) * p.ldb_b + Kb));

    AccT acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    OpA a;
    OpB b;
    const int KT = (Kb + ROWB - 1) / ROWB;
    a.load(ra, tid, 0, p.lda_b, Kb);
    b.load(rb, tid, 0, p.ldb_b, Kb);
    a.store(lds, tid);
    b.store(lds + OpA::BYTES, tid);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
    int cur = 0;
    for (int kt = 0; kt < KT; ++kt) {
        // loads past the last step are out of range: they return zeros and touch no memory
        a.load(ra, tid, kt + 1, p.lda_b, Kb);
        b.load(rb, tid, kt + 1, p.ldb_b, Kb);
        const char *sa = lds + cur, *sb = lds + cur + OpA::BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4 af[MI], bf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = OpA::frag(sa, wm * WTM + i * 32, kk, lane);
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[j] = OpB::frag(sb, wn * WTN + j * 32, kk, lane);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j] = Acc<INT8>::mma(af[i], bf[j], acc[i][j]);
        }
        const int nxt = cur ^ STAGE;
        a.store(lds + nxt, tid);                       // the buffer multiplied one barrier ago
        b.store(lds + nxt + OpA::BYTES, tid);
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
        cur = nxt;
    }

    using OutT = typename std::conditional<INT8, int, float>::type;
    OutT *C = (OutT *)p.C + batch * p.strideC;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
            store_block32<INT8>(acc[i][j], C, p.ldc, m0 + wm * WTM + i * 32, n0 + wn * WTN + j * 32, lane, p.M, p.N,
                                p.alpha, p.beta);
}

// ------------------------------------------------------------------------------------ host side

template <bool INT8>
bool oc_operand_ok(const void *base, int64_t s_outer, int64_t s_k, int64_t outer, int64_t K, int64_t stride, int tile,
                   bool *is_oc)
{
    const int64_t esz = INT8 ? 1 : 2;
    if (((uintptr_t)base % 16) != 0 || (stride * esz) % 16 != 0) return false;
    if (s_k == 1) {
        // contiguous along K
        *is_oc = false;
        if ((s_outer * esz) % 16 != 0 || (K * esz) % 16 != 0) return false;
        return (tile - 1) * s_outer * esz + K * esz < 0x7fffffffLL;
    }
    if (s_outer == 1) {
        *is_oc = true;
        if ((s_k * esz) % 16 != 0 || (outer * esz) % 16 != 0) return false;
        return (K + 2 * (int64_t)(ROWB / esz)) * s_k * esz + outer * esz < 0x7fffffffLL;
    }
    return false;
}

template <bool INT8, int BM, int BN, int WM, int WN>
bool oc_can_run(const Problem &q)
{
    if (q.c_plane) return false;                          // planar output: the general and direct-to-LDS kernels only
    if (q.in_type != (INT8 ? XP_I8 : XP_BF16) || q.conv) return false;
    if (q.K <= 0 || q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.K > 0x3fffffffLL || q.batch > 65535) return false;
    bool a_oc, b_oc;
    if (!oc_operand_ok<INT8>(q.A, q.a_sm, q.a_sk, q.M, q.K, q.strideA, BM, &a_oc)) return false;
    if (!oc_operand_ok<INT8>(q.B, q.b_sn, q.b_sk, q.N, q.K, q.strideB, BN, &b_oc)) return false;
    if (!a_oc && !b_oc) return false;                 // both along K: the other MFMA kernels serve that
    return ((q.M + BM - 1) / BM) * ((q.N + BN - 1) / BN) <= 0x7fffffffLL;
}

template <bool INT8, int BM, int BN, int WM, int WN>
hipError_t oc_launch(const Problem &q)
{
    const int64_t esz = INT8 ? 1 : 2;
    bool a_oc = false, b_oc = false;
    oc_operand_ok<INT8>(q.A, q.a_sm, q.a_sk, q.M, q.K, q.strideA, BM, &a_oc);
    oc_operand_ok<INT8>(q.B, q.b_sn, q.b_sk, q.N, q.K, q.strideB, BN, &b_oc);
    OcParams p;
    p.A = (const char *)q.A; p.B = (const char *)q.B; p.C = (char *)q.C;
    p.M = (int)q.M; p.N = (int)q.N; p.K = (int)q.K;
    p.lda_b = (a_oc ? q.a_sk : q.a_sm) * esz;
    p.ldb_b = (b_oc ? q.b_sk : q.b_sn) * esz;
    p.ldc = q.ldc;
    p.strideA_b = q.strideA * esz; p.strideB_b = q.strideB * esz; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    const int tiles_m = (int)((q.M + BM - 1) / BM);
    p.tiles_n = (int)((q.N + BN - 1) / BN);
    const dim3 grid((unsigned)(tiles_m * p.tiles_n), (unsigned)q.batch), block(WM * WN * 64);
    if (a_oc && b_oc) hipLaunchKernelGGL((oc_kernel<INT8, BM, BN, WM, WN, true, true>), grid, block, 0, q.stream, p);
    else if (a_oc) hipLaunchKernelGGL((oc_kernel<INT8, BM, BN, WM, WN, true, false>), grid, block, 0, q.stream, p);
    else hipLaunchKernelGGL((oc_kernel<INT8, BM, BN, WM, WN, false, true>), grid, block, 0, q.stream, p);
    return hipGetLastError();
}

template <int BM, int BN, int WM, int WN>
double oc_cost(const Problem &q)
{
    const int lds = 2 * (BM + BN) * (ROWB + 8);
    return tile_cost_us(q, BM, BN, lds, WM * WN * 64, BM * BN >= 128 * 128 ? 0.25 : 0.18, q.in_type == XP_I8 ? 1 : 2);
}

#define XP_OC_VARIANT(NAME, TYPESTR, INT8, BM, BN, WM, WN)                                                   \
    const Variant NAME = {TYPESTR " " #BM "x" #BN "x128B waves " #WM "x" #WN " k-group-interleaved mfma32", \
                          oc_can_run<INT8, BM, BN, WM, WN>, oc_launch<INT8, BM, BN, WM, WN>, oc_cost<BM, BN, WM, WN>};

XP_OC_VARIANT(kBfOc128x128, "bf16", false, 128, 128, 2, 2)
XP_OC_VARIANT(kBfOc128x64, "bf16", false, 128, 64, 4, 1)
XP_OC_VARIANT(kBfOc64x64, "bf16", false, 64, 64, 2, 2)
XP_OC_VARIANT(kI8Oc128x128, "i8", true, 128, 128, 2, 2)
XP_OC_VARIANT(kI8Oc128x64, "i8", true, 128, 64, 4, 1)
XP_OC_VARIANT(kI8Oc64x64, "i8", true, 64, 64, 2, 2)

}  // namespace

int oc_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) { out[0] = &kBfOc128x128; out[1] = &kBfOc128x64; out[2] = &kBfOc64x64; return 3; }
    if (in_type == XP_I8) { out[0] = &kI8Oc128x128; out[1] = &kI8Oc128x64; out[2] = &kI8Oc64x64; return 3; }
    return 0;
}

}  // namespace xp
