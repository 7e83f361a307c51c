// Ping-pong MFMA kernel for large GEMMs with both operands contiguous along K (bf16 and int8;
// Table 5 of the paper: GEMM, Batch GEMM): 256 x 256 tile of C per workgroup, 8 waves, each owning a
// 128 x 64 sub-tile, K walked in steps of 128 bytes per row through two LDS buffers that are filled
// by direct global -> LDS loads.
//
// What differs from the other direct-to-LDS kernels is the schedule (the Pipeline pass of Table 4
// taken one step further).  The two waves that share a SIMD never do the same thing at the same
// time: waves 0-3 ("early") and waves 4-7 ("late", one per SIMD each) alternate between
//   MEMORY(k):   read all fragments of K step k from LDS into registers (24 x 16 bytes per lane);
//                the early waves also issue every global load of K step k+1
//   COMPUTE(k):  the 32 (32x32x16) or 64 (16x16x32) MFMAs of K step k, back to back, at raised
//                wave priority
// separated by workgroup barriers, the late waves one phase behind the early ones:
//
//   slot      0        1        2        3        4     ...
//   early   MEM(0)  CMP(0)   MEM(1)   CMP(1)   MEM(2)
//   late      -     MEM(0)   CMP(0)   MEM(1)   CMP(1)
//
// so that in every slot one wave per SIMD feeds the MFMA pipe while the other one moves data, and
// neither LDS latency nor global latency is ever on the MFMA wave's path.  K step k+1 is loaded
// (slot 2k) into the buffer whose last reader (late MEM(k-1), slot 2k-1) has passed a barrier, and
// must have landed two slots later (early MEM(k+1), slot 2k+2): the early waves wait for their own
// loads at the end of CMP(k).  Loads past the end of K or of the matrix are out of range for the
// buffer resource: zeros are written to LDS, no memory is touched, no conditionals are needed.
#include "xp_internal.hpp"
#include "xp_epilogue.hpp"

#include <cstdlib>
#include <type_traits>

namespace xp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int BM = 256, BN = 256, RB = 128;
constexpr int WTM = 128, WTN = 64;                    // wave sub-tile: waves 2 (M) x 4 (N)
constexpr int STAGE = (BM + BN) * RB;
constexpr unsigned OOB = 0x80000000u;

struct PpParams {
    const char *A, *B;
    char *C;
    int M, N, Kb, KT;
    long long lda_b, ldb_b, ldc;
    long long strideA_b, strideB_b, strideC;
    float alpha, beta;
    int tiles_m, tiles_n, group_m;
};

// Chunk swizzle: a per-row XOR of the 16-byte chunk index such that the 16 lanes that one pass of a
// 128-bit LDS read serves (lane quads of equal bit parity within half a wave, as measured) hit 16
// different bank groups, for 32-row and for 16-row MFMA blocks respectively.
template <int MF> __device__ __forceinline__ int swz(int row)
{
    if constexpr (MF == 32) return (row & 7) ^ ((row >> 3) & 1);
    else return row & 6;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// workgroup barrier that the compiler may move neither memory accesses nor any other instruction across
__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <bool INT8, int MF> struct Mma;
template <> struct Mma<false, 32> {
    typedef f32x16 acc_t;
    __device__ static __forceinline__ acc_t run(u32x4 a, u32x4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                       c, 0, 0, 0);
    }
};
template <> struct Mma<true, 32> {
    typedef i32x16 acc_t;
    __device__ static __forceinline__ acc_t run(u32x4 a, u32x4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b),
                                                     c, 0, 0, 0);
    }
};
template <> struct Mma<false, 16> {
    typedef f32x4 acc_t;
    __device__ static __forceinline__ acc_t run(u32x4 a, u32x4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                       c, 0, 0, 0);
    }
};
template <> struct Mma<true, 16> {
    typedef i32x4 acc_t;
    __device__ static __forceinline__ acc_t run(u32x4 a, u32x4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b),
                                                     c, 0, 0, 0);
    }
};

template <bool INT8, int MF>
__global__ __launch_bounds__(512) void pp_kernel(PpParams p)
{
    using AccT = typename Mma<INT8, MF>::acc_t;
    constexpr int MI = WTM / MF, NI = WTN / MF;       // MFMA blocks per wave
    constexpr int PH = RB * MF / 1024;                // MFMA sub-steps per K step (one consumes 1024/MF bytes of a row)
    constexpr int NACC = MF == 32 ? 16 : 4;
    __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool early = wave < 4;                      // waves w and w+4 share a SIMD
    const int wm = wave >> 2, wn = wave & 3;

    // workgroup -> tile: one XCD (workgroup id mod 8) owns a run of consecutive tiles, walked in
    // groups of group_m tile-rows, so that the tiles sharing an L2 share A and B panels
    int bid = blockIdx.x;
    const int nb = p.tiles_m * p.tiles_n;
    if ((nb & 7) == 0) bid = (bid & 7) * (nb >> 3) + (bid >> 3);
    const int gsz = p.group_m * p.tiles_n;
    const int g = bid / gsz, first_m = g * p.group_m;
    const int gm = min(p.tiles_m - first_m, p.group_m);
    const int tm = first_m + (bid % gsz) % gm, tn = (bid % gsz) / gm;
    const int m0 = tm * BM, n0 = tn * BN;
    const long long batch = blockIdx.y;

    // ---- global -> LDS loads (early waves only).  One wave-level load fills the 1024 LDS bytes of
    // an 8-row block, lane l at row l/8, position l%8; the lane fetches the chunk whose swizzled
    // position that is.  Wave w loads row blocks w, w+4, w+8, ... of A and of B: the row of slot i
    // is (w + 4i)*8 + l/8, so the swizzle term and the chunk are the same for every slot.
    const __amdgpu_buffer_rsrc_t ra =
        make_rsrc(p.A + batch * p.strideA_b + (long long)m0 * p.lda_b,
                  (unsigned)((long long)(min(p.M - m0, BM) - 1) * p.lda_b + p.Kb));
    const __amdgpu_buffer_rsrc_t rb =
        make_rsrc(p.B + batch * p.strideB_b + (long long)n0 * p.ldb_b,
                  (unsigned)((long long)(min(p.N - n0, BN) - 1) * p.ldb_b + p.Kb));
    const int lrow = (wave & 3) * 8 + (lane >> 3);
    const int lchunk = ((lane & 7) ^ swz<MF>(lrow)) << 4;
    const unsigned a_off0 = (unsigned)(lrow * p.lda_b) + lchunk, b_off0 = (unsigned)(lrow * p.ldb_b) + lchunk;
    const unsigned a_step = (unsigned)(32 * p.lda_b), b_step = (unsigned)(32 * p.ldb_b);
    auto issue = [&](int kt, int stage_off) {
        const int kb = kt * RB;
        const bool dead = kb + lchunk >= p.Kb;          // chunk past the end of K
#pragma unroll
        for (int i = 0; i < BM / 32; ++i) {
            const unsigned off = dead ? OOB : a_off0 + i * a_step;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void *)(lds + stage_off + ((wave & 3) + 4 * i) * 1024), 16,
                                                     off, kb, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < BN / 32; ++i) {
            const unsigned off = dead ? OOB : b_off0 + i * b_step;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rb, (lds_void *)(lds + stage_off + BM * RB + ((wave & 3) + 4 * i) * 1024), 16, off, kb, 0, 0);
        }
    };

    // ---- fragments: lane l reads row l % MF of an MF-row block, chunk (64/MF)*kk + l/MF
    const int frow = lane & (MF - 1), fch = lane / MF, fsw = swz<MF>(frow);
    int fa[PH], fb[PH];
#pragma unroll
    for (int kk = 0; kk < PH; ++kk) {
        const int c = (((64 / MF) * kk + fch) ^ fsw) << 4;
        fa[kk] = (wm * WTM + frow) * RB + c;
        fb[kk] = BM * RB + (wn * WTN + frow) * RB + c;
    }
    u32x4 af[PH][MI], bf[PH][NI];
    auto memory = [&](int stage_off) {
#pragma unroll
        for (int kk = 0; kk < PH; ++kk) {
#pragma unroll
            for (int i = 0; i < MI; ++i) af[kk][i] = *(const u32x4 *)(lds + stage_off + fa[kk] + i * MF * RB);
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[kk][j] = *(const u32x4 *)(lds + stage_off + fb[kk] + j * MF * RB);
        }
    };

    AccT acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < NACC; ++v) acc[i][j][v] = 0;
    auto compute = [&]() {
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int kk = 0; kk < PH; ++kk)
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    // 16x16 blocks are computed transposed so that a lane holds 4 consecutive columns of C
                    if constexpr (MF == 32) acc[i][j] = Mma<INT8, 32>::run(af[kk][i], bf[kk][j], acc[i][j]);
                    else acc[i][j] = Mma<INT8, 16>::run(bf[kk][j], af[kk][i], acc[i][j]);
                }
        __builtin_amdgcn_s_setprio(0);
    };

    // ---- schedule.  Every wave executes exactly 2*KT + 1 barriers (KT >= 1 is checked on the host).
    const int KT = p.KT;
    if (KT < 1) return;
    if (early) {
        issue(0, 0);
        __builtin_amdgcn_s_waitcnt(0x0070);             // vmcnt(0) lgkmcnt(0): K step 0 has landed
        wg_barrier();                                   // B(0)
        int cur = 0;
        for (int k = 0; k < KT; ++k) {
            issue(k + 1, cur ^ STAGE);                  // last read by the late waves one barrier ago
            memory(cur);
            __builtin_amdgcn_s_waitcnt(0xc07f);         // lgkmcnt(0): fragments are in registers
            wg_barrier();                               // B(2k+1)
            compute();
            __builtin_amdgcn_s_waitcnt(0x0070);         // K step k+1 has landed
            wg_barrier();                               // B(2k+2)
            cur ^= STAGE;
        }
    } else {
        wg_barrier();                                   // B(0)
        wg_barrier();                                   // B(1)
        int cur = 0;
        for (int k = 0; k < KT; ++k) {
            memory(cur);
            __builtin_amdgcn_s_waitcnt(0xc07f);
            wg_barrier();                               // B(2k+2)
            compute();
            if (k + 1 < KT) wg_barrier();               // B(2k+3)
            cur ^= STAGE;
        }
    }

    // ---- epilogue
    using OutT = typename std::conditional<INT8, int, float>::type;
    OutT *C = (OutT *)p.C + batch * p.strideC;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            if constexpr (MF == 32)
                store_block32<INT8>(acc[i][j], C, p.ldc, m0 + wm * WTM + i * 32, n0 + wn * WTN + j * 32, lane, p.M, p.N,
                                    p.alpha, p.beta);
            else
                store_block16t<INT8>(acc[i][j], C, p.ldc, m0 + wm * WTM + i * 16, n0 + wn * WTN + j * 16, lane, p.M, p.N,
                                     p.alpha, p.beta);
        }
}

// ------------------------------------------------------------------------------------ host side

template <bool INT8>
bool pp_can_run(const Problem &q)
{
    if (q.c_plane) return false;                          // planar output: the general and direct-to-LDS kernels only
    const int64_t esz = INT8 ? 1 : 2;
    if (q.in_type != (INT8 ? XP_I8 : XP_BF16) || q.conv) return false;
    if (q.K <= 0 || (q.K * esz) % 16 != 0) return false;
    if (q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.K * esz > 0x3fffffffLL || q.batch > 65535) return false;
    if (q.a_sk != 1 || q.b_sk != 1) return false;
    if ((q.a_sm * esz) % 16 != 0 || (q.b_sn * esz) % 16 != 0) return false;
    if (((uintptr_t)q.A % 16) != 0 || ((uintptr_t)q.B % 16) != 0) return false;
    if ((q.strideA * esz) % 16 != 0 || (q.strideB * esz) % 16 != 0) return false;
    if (BM * q.a_sm * esz + q.K * esz >= 0x7fffffffLL || BN * q.b_sn * esz + q.K * esz >= 0x7fffffffLL) return false;
    return ((q.M + BM - 1) / BM) * ((q.N + BN - 1) / BN) <= 0x7fffffffLL;
}

template <bool INT8, int MF>
hipError_t pp_launch(const Problem &q)
{
    const int64_t esz = INT8 ? 1 : 2;
    PpParams p;
    p.A = (const char *)q.A; p.B = (const char *)q.B; p.C = (char *)q.C;
    p.M = (int)q.M; p.N = (int)q.N;
    p.Kb = (int)(q.K * esz);
    p.KT = (p.Kb + RB - 1) / RB;
    p.lda_b = q.a_sm * esz; p.ldb_b = q.b_sn * esz; p.ldc = q.ldc;
    p.strideA_b = q.strideA * esz; p.strideB_b = q.strideB * esz; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    p.tiles_m = (int)((q.M + BM - 1) / BM);
    p.tiles_n = (int)((q.N + BN - 1) / BN);
    // tile-rows per raster group; XP_GROUP_M overrides it for tuning experiments
    static const int env_group_m = [] { const char *e = getenv("XP_GROUP_M"); return e ? atoi(e) : 0; }();
    p.group_m = env_group_m > 0 ? env_group_m : 4;
    hipLaunchKernelGGL((pp_kernel<INT8, MF>), dim3((unsigned)(p.tiles_m * p.tiles_n), (unsigned)q.batch), dim3(512), 0,
                       q.stream, p);
    return hipGetLastError();
}

template <bool INT8, int MF>
double pp_cost(const Problem &q)
{
    // ahead of the plain direct-to-LDS kernel once the grid is several rounds deep (swept at 8192^3)
    return tile_cost_us(q, BM, BN, 2 * STAGE, 512, MF == 16 ? 0.565 : 0.525, INT8 ? 1 : 2);
}

const Variant kBfPp32 = {"bf16 256x256x128B waves 2x4 ring 2 ping-pong direct-to-lds mfma32", pp_can_run<false>,
                         pp_launch<false, 32>, pp_cost<false, 32>};
const Variant kBfPp16 = {"bf16 256x256x128B waves 2x4 ring 2 ping-pong direct-to-lds mfma16", pp_can_run<false>,
                         pp_launch<false, 16>, pp_cost<false, 16>};
const Variant kI8Pp32 = {"i8 256x256x128B waves 2x4 ring 2 ping-pong direct-to-lds mfma32", pp_can_run<true>,
                         pp_launch<true, 32>, pp_cost<true, 32>};
const Variant kI8Pp16 = {"i8 256x256x128B waves 2x4 ring 2 ping-pong direct-to-lds mfma16", pp_can_run<true>,
                         pp_launch<true, 16>, pp_cost<true, 16>};

}  // namespace

int pp_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) { out[0] = &kBfPp32; out[1] = &kBfPp16; return 2; }
    if (in_type == XP_I8) { out[0] = &kI8Pp32; out[1] = &kI8Pp16; return 2; }
    return 0;
}

}  // namespace xp
