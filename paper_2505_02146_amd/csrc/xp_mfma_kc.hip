// Tuned MFMA kernels for operands that are contiguous along K ("kc"): bf16 x bf16 -> fp32 and
// int8 x int8 -> int32 GEMM, strided-batched GEMM, and the implicit-GEMM form of the NHWC
// convolution (Table 5 of the paper: GEMM, Batch GEMM, Conv2D NHWC; the contraction uses the
// matrix-core MFMA instructions of the kind Table 1 names for AMD hardware).
//
// Structure of one workgroup (one BM x BN tile of C, K walked in steps of 128 bytes per row):
//   global -> registers -> LDS   16-byte loads through a buffer resource whose range check
//                                zero-fills rows past the edge of the matrix; rows are stored
//                                in LDS 128 bytes apart with the 16-byte chunk index XOR-ed by a
//                                function of the row, so that the MFMA fragment reads (32 rows x
//                                one chunk) and the staging writes are both bank-conflict free
//   LDS -> fragments -> MFMA     32x32x16 (bf16) or 32x32x32 (int8) MFMA, WM x WN waves, each
//                                owning a (BM/WM) x (BN/WN) sub-tile held in accumulators
//   software pipeline            NSTAGE LDS buffers; the tile for step t+1 is written to LDS
//                                and the global loads for step t+2 are issued while step t is
//                                being multiplied; one workgroup barrier per step
//   epilogue                     alpha/beta in registers, 128-byte row segments stored directly
//
// The im2col view of the convolution only changes how a staging thread turns (tile row, K offset)
// into a global address: row m = (n, p, q), K offset = (r, s, c); taps that fall into the zero
// padding are redirected past the end of the buffer range so that the load returns zeros.
#include "xp_internal.hpp"
#include "xp_epilogue.hpp"

#include <cstdio>
#include <cstdlib>
#include <type_traits>

namespace xp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWB = 128;                 // bytes of K per tile row and step
constexpr unsigned OOB = 0x80000000u;     // byte offset that is outside every buffer range used here

struct KcParams {
    const char *A, *B;
    char *C;
    int M, N;
    int Kb;                               // K in bytes
    int KT;                               // number of K steps
    long long lda_b, ldb_b;               // row pitches in bytes
    long long ldc;                        // elements
    long long strideA_b, strideB_b, strideC;
    float alpha, beta;
    int tiles_m, tiles_n, group_m;
    // convolution view
    unsigned in_bytes;
    int H, W, Cin_b, S, PQ, Q, sh, sw, ph, pw;
};

template <int BM_, int BN_, int WM_, int WN_, int NSTAGE_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NSTAGE = NSTAGE_;
    static constexpr int NT = WM * WN * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;      // wave sub-tile
    static constexpr int MI = WTM / 32, NI = WTN / 32;      // 32x32 MFMA blocks per wave
    static constexpr int LA = BM * 8 / NT, LB = BN * 8 / NT;  // 16-byte loads per thread and step
    static constexpr int STAGE = (BM + BN) * ROWB;
    static constexpr int LDS = NSTAGE * STAGE;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave sub-tile must be whole MFMA blocks");
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "staging must divide evenly");
    static_assert(LDS <= 160 * 1024, "LDS budget of one compute unit");
    static_assert(NSTAGE == 2, "the pipeline ping-pongs between two LDS buffers");
};

// chunk swizzle: a per-row XOR of the 16-byte chunk index; distinct for 8 consecutive rows and
// for same-parity rows of 16 consecutive rows, which covers 128-byte and 256-byte bank widths
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

template <bool INT8, class T, bool CONV>
__global__ __launch_bounds__(T::NT) void kc_kernel(KcParams p)
{
    using AccT = typename Acc<INT8>::type;
    __shared__ __attribute__((aligned(16))) char lds[T::LDS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / T::WN, wn = wave % T::WN;

    // ---- workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its own
    // L2); renumber so that one XCD owns a run of consecutive tile numbers, then walk the tiles
    // in groups of group_m tile-rows so that the run is a compact block sharing A and B panels.
    int bid = blockIdx.x;
    const int nb = p.tiles_m * p.tiles_n;
    if ((nb & 7) == 0) bid = (bid & 7) * (nb >> 3) + (bid >> 3);
    const int gsz = p.group_m * p.tiles_n;
    const int g = bid / gsz, first_m = g * p.group_m;
    const int gm = min(p.tiles_m - first_m, p.group_m);
    const int tm = first_m + (bid % gsz) % gm, tn = (bid % gsz) / gm;
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const long long batch = blockIdx.y;

    // ---- buffer resources.  The range ends after the last valid row, so that every row past
    // the edge reads as zeros; the K offset of a step travels in the scalar offset (not range
    // checked), and chunks past K are redirected to OOB explicitly.
    const int rows_a = min(p.M - m0, T::BM), rows_b = min(p.N - n0, T::BN);
    __amdgpu_buffer_rsrc_t ra, rb;
    if constexpr (CONV) {
        ra = make_rsrc(p.A, p.in_bytes);
    } else {
        ra = make_rsrc(p.A + batch * p.strideA_b + (long long)m0 * p.lda_b,
                       (unsigned)((long long)(rows_a - 1) * p.lda_b + p.Kb));
    }
    rb = make_rsrc(p.B + batch * p.strideB_b + (long long)n0 * p.ldb_b,
                   (unsigned)((long long)(rows_b - 1) * p.ldb_b + p.Kb));

    // ---- per-thread staging slots: slot i covers tile row (tid + i*NT)/8, chunk (tid + i*NT)%8
    unsigned a_off[T::LA], b_off[T::LB];
    int a_lds[T::LA], b_lds[T::LB];
    int a_h0[CONV ? T::LA : 1], a_w0[CONV ? T::LA : 1];
    const int chunk = tid & 7;
#pragma unroll
    for (int i = 0; i < T::LA; ++i) {
        const int row = (tid + i * T::NT) >> 3;
        a_lds[i] = row * ROWB + ((chunk ^ swz(row)) << 4);
        if constexpr (CONV) {
            const int m = m0 + row;
            if (m < p.M) {
                const int n = m / p.PQ, pq = m % p.PQ;
                const int op = pq / p.Q, oq = pq % p.Q;
                a_h0[i] = op * p.sh - p.ph;
                a_w0[i] = oq * p.sw - p.pw;
                a_off[i] = (unsigned)n * (unsigned)(p.H * p.W) * (unsigned)p.Cin_b + (chunk << 4);
            } else {
                a_h0[i] = -0x40000000;      // never inside the image
                a_w0[i] = 0;
                a_off[i] = 0;
            }
        } else {
            a_off[i] = (unsigned)(row * p.lda_b) + (chunk << 4);
        }
    }
#pragma unroll
    for (int i = 0; i < T::LB; ++i) {
        const int row = (tid + i * T::NT) >> 3;
        b_lds[i] = T::BM * ROWB + row * ROWB + ((chunk ^ swz(row)) << 4);
        b_off[i] = (unsigned)(row * p.ldb_b) + (chunk << 4);
    }

    // ---- fragment read addresses: lane l reads row (l & 31) of a 32-row block, chunk 2*kk + (l >> 5)
    const int frow = lane & 31, fhi = lane >> 5;
    const int fsw = swz(frow);              // blocks start at multiples of 32 rows: same swizzle
    int fa[4], fb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int c = ((2 * kk + fhi) ^ fsw) << 4;
        fa[kk] = (wm * T::WTM + frow) * ROWB + c;
        fb[kk] = T::BM * ROWB + (wn * T::WTN + frow) * ROWB + c;
    }

    AccT acc[T::MI][T::NI];
#pragma unroll
    for (int i = 0; i < T::MI; ++i)
#pragma unroll
        for (int j = 0; j < T::NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    u32x4 ga[T::LA], gb[T::LB];

    // conv: the K offset of a step is (tap, c0); it advances without divisions
    int tap_r = 0, tap_s = 0, c0_b = 0;

    // One staging slot = one 16-byte chunk per thread: slots [0, LA) belong to A, the rest to B.
    // Loads past the last K step are redirected out of range (they return zeros without touching
    // memory), so the pipeline below needs no conditionals.
    constexpr int NSLOT = T::LA + T::LB;
    auto kmask_of = [&](int kt) -> unsigned {
        const int kb = kt * ROWB;
        return (kb + (chunk << 4) >= p.Kb) ? OOB : 0u;
    };
    auto load_slot = [&](int i, int kt, unsigned kmask) {
        const int kb = kt * ROWB;
        if (i < T::LA) {
            unsigned off;
            int soff;
            if constexpr (CONV) {
                const int h = a_h0[i] + tap_r, w = a_w0[i] + tap_s;
                const bool ok = (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W;
                off = ok ? a_off[i] + (unsigned)(h * p.W + w) * (unsigned)p.Cin_b : OOB;
                soff = c0_b;
            } else {
                off = a_off[i];
                soff = kb;
            }
            ga[i] = __builtin_amdgcn_raw_buffer_load_b128(ra, off | kmask, soff, 0);
        } else {
            gb[i - T::LA] = __builtin_amdgcn_raw_buffer_load_b128(rb, b_off[i - T::LA] | kmask, kb, 0);
        }
    };
    auto advance_tap = [&]() {
        if constexpr (CONV) {
            c0_b += ROWB;
            if (c0_b >= p.Cin_b) {
                c0_b = 0;
                if (++tap_s == p.S) { tap_s = 0; ++tap_r; }
            }
        }
    };
    auto store_slot = [&](int i, int stage_off) {
        if (i < T::LA) *(u32x4 *)(lds + stage_off + a_lds[i]) = ga[i];
        else *(u32x4 *)(lds + stage_off + b_lds[i - T::LA]) = gb[i - T::LA];
    };
    auto read_frags = [&](int stage_off, int kk, u32x4 (&af)[T::MI], u32x4 (&bf)[T::NI]) {
#pragma unroll
        for (int i = 0; i < T::MI; ++i) af[i] = *(const u32x4 *)(lds + stage_off + fa[kk] + i * 32 * ROWB);
#pragma unroll
        for (int j = 0; j < T::NI; ++j) bf[j] = *(const u32x4 *)(lds + stage_off + fb[kk] + j * 32 * ROWB);
    };
    auto mma_all = [&](const u32x4 (&af)[T::MI], const u32x4 (&bf)[T::NI]) {
#pragma unroll
        for (int i = 0; i < T::MI; ++i)
#pragma unroll
            for (int j = 0; j < T::NI; ++j) acc[i][j] = Acc<INT8>::mma(af[i], bf[j], acc[i][j]);
    };

    // ---- pipeline.  Per K step (4 MFMA sub-steps kk of 32 bytes of K each):
    //   sub-steps 0..2: read the fragments of sub-step kk+1, write a third of the staged tile of
    //                   step kt+1 to the other LDS buffer and re-issue those slots' global loads
    //                   for step kt+2, then multiply sub-step kk
    //   sub-step 3:     wait for this wave's LDS traffic, workgroup barrier, read the fragments of
    //                   sub-step 0 of the next buffer, then multiply sub-step 3 (whose fragments
    //                   were read before the barrier), so that the barrier is covered by MFMA work
    // Fragments ping-pong between two register sets (X, Y).
    const int KT = p.KT;
    if (KT > 0) {
        u32x4 xa[T::MI], xb[T::NI], ya[T::MI], yb[T::NI];
        {
            const unsigned km = kmask_of(0);
#pragma unroll
            for (int i = 0; i < NSLOT; ++i) load_slot(i, 0, km);
            advance_tap();
#pragma unroll
            for (int i = 0; i < NSLOT; ++i) store_slot(i, 0);
            const unsigned km1 = kmask_of(1);
#pragma unroll
            for (int i = 0; i < NSLOT; ++i) load_slot(i, 1, km1);
            advance_tap();
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);     // lgkmcnt(0): this wave's LDS writes have landed
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, xa, xb);
        constexpr int S0 = (NSLOT + 2) / 3, S1 = (2 * NSLOT + 2) / 3;
        // One K step.  The buffer that is read (CUR) is a template constant, so every LDS address is a
        // register plus an immediate; CHECK: the step loaded here (kt + 2) may reach past K, so each
        // lane masks its chunk.  The main part of the loop needs neither: vector instructions do not
        // overlap with matrix instructions on a SIMD, so address adds and masks there are MFMA time lost.
        auto step = [&](int kt, auto cur_c, auto check_c) {
            constexpr int cur = decltype(cur_c)::value ? T::STAGE : 0, nxt = cur ^ T::STAGE;
            constexpr bool CHECK = decltype(check_c)::value;
            unsigned km = 0u;
            if constexpr (CHECK) km = kmask_of(kt + 2);
            // sub-step 0
            read_frags(cur, 1, ya, yb);
#pragma unroll
            for (int i = 0; i < S0; ++i) store_slot(i, nxt);
#pragma unroll
            for (int i = 0; i < S0; ++i) load_slot(i, kt + 2, km);
            __builtin_amdgcn_sched_barrier(0);
            mma_all(xa, xb);
            __builtin_amdgcn_sched_barrier(0);
            // sub-step 1
            read_frags(cur, 2, xa, xb);
#pragma unroll
            for (int i = S0; i < S1; ++i) store_slot(i, nxt);
#pragma unroll
            for (int i = S0; i < S1; ++i) load_slot(i, kt + 2, km);
            __builtin_amdgcn_sched_barrier(0);
            mma_all(ya, yb);
            __builtin_amdgcn_sched_barrier(0);
            // sub-step 2
            read_frags(cur, 3, ya, yb);
#pragma unroll
            for (int i = S1; i < NSLOT; ++i) store_slot(i, nxt);
#pragma unroll
            for (int i = S1; i < NSLOT; ++i) load_slot(i, kt + 2, km);
            advance_tap();
            __builtin_amdgcn_sched_barrier(0);
            mma_all(xa, xb);
            __builtin_amdgcn_sched_barrier(0);
            // sub-step 3
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_s_barrier();
            read_frags(nxt, 0, xa, xb);          // garbage after the last step, never multiplied
            __builtin_amdgcn_sched_barrier(0);
            mma_all(ya, yb);
            __builtin_amdgcn_sched_barrier(0);
        };
        const int whole = p.Kb / ROWB - 2;       // steps kt < whole load a step that lies wholly inside K
        int kt = 0;
        for (; kt + 1 < whole; kt += 2) {
            step(kt, std::false_type{}, std::false_type{});
            step(kt + 1, std::true_type{}, std::false_type{});
        }
        for (; kt + 1 < KT; kt += 2) {
            step(kt, std::false_type{}, std::true_type{});
            step(kt + 1, std::true_type{}, std::true_type{});
        }
        if (kt < KT) step(kt, std::false_type{}, std::true_type{});
    }

    // ---- epilogue
    using OutT = typename std::conditional<INT8, int, float>::type;
    OutT *C = (OutT *)p.C + batch * p.strideC;
#pragma unroll
    for (int i = 0; i < T::MI; ++i)
#pragma unroll
        for (int j = 0; j < T::NI; ++j)
            store_block32<INT8>(acc[i][j], C, p.ldc, m0 + wm * T::WTM + i * 32, n0 + wn * T::WTN + j * 32, lane, p.M, p.N,
                                p.alpha, p.beta);
}

// ------------------------------------------------------------------------------------ host side

template <bool INT8>
bool kc_can_run_common(const Problem &q, int BM, int BN)
{
    if (q.c_plane) return false;                          // planar output: the general and direct-to-LDS kernels only
    const int64_t esz = INT8 ? 1 : 2;
    if (q.in_type != (INT8 ? XP_I8 : XP_BF16)) return false;
    if (q.K <= 0) return false;
    if ((q.K * esz) % 16 != 0) return false;
    if (q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.K * esz > 0x7fffffffLL) return false;
    if (q.batch > 65535) return false;
    // B: contiguous along K, 16-byte aligned rows
    if (q.b_sk != 1 || (q.b_sn * esz) % 16 != 0 || ((uintptr_t)q.B % 16) != 0) return false;
    if ((q.strideB * esz) % 16 != 0) return false;
    if ((BN - 1) * q.b_sn * esz + q.K * esz >= 0x7fffffffLL) return false;
    if (q.conv) {
        if (INT8) return false;
        const int64_t in_bytes = (q.M / (q.P * q.Q)) * q.H * q.W * q.Cin * esz;
        if (in_bytes >= 0x7fffffffLL) return false;
        if ((q.Cin * esz) % ROWB != 0) return false;       // a K step never straddles a filter tap
        if (((uintptr_t)q.A % 16) != 0) return false;
    } else {
        if (q.a_sk != 1 || (q.a_sm * esz) % 16 != 0 || ((uintptr_t)q.A % 16) != 0) return false;
        if ((q.strideA * esz) % 16 != 0) return false;
        if ((BM - 1) * q.a_sm * esz + q.K * esz >= 0x7fffffffLL) return false;
    }
    const int64_t tiles = ((q.M + BM - 1) / BM) * ((q.N + BN - 1) / BN);
    return tiles <= 0x7fffffffLL;
}

template <bool INT8, class T>
hipError_t kc_launch(const Problem &q)
{
    const int64_t esz = INT8 ? 1 : 2;
    KcParams p;
    p.A = (const char *)q.A; p.B = (const char *)q.B; p.C = (char *)q.C;
    p.M = (int)q.M; p.N = (int)q.N;
    p.Kb = (int)(q.K * esz);
    p.KT = (p.Kb + ROWB - 1) / ROWB;
    p.lda_b = q.a_sm * esz; p.ldb_b = q.b_sn * esz;
    p.ldc = q.ldc;
    p.strideA_b = q.strideA * esz; p.strideB_b = q.strideB * esz; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    p.tiles_m = (int)((q.M + T::BM - 1) / T::BM);
    p.tiles_n = (int)((q.N + T::BN - 1) / T::BN);
    // tile-rows per raster group; XP_GROUP_M overrides it for tuning experiments
    static const int env_group_m = [] { const char *e = getenv("XP_GROUP_M"); return e ? atoi(e) : 0; }();
    p.group_m = env_group_m > 0 ? env_group_m : 4;
    p.in_bytes = 0; p.H = p.W = p.Cin_b = p.S = p.PQ = p.Q = p.sh = p.sw = p.ph = p.pw = 0;
    if (q.conv) {
        p.in_bytes = (unsigned)((q.M / (q.P * q.Q)) * q.H * q.W * q.Cin * esz);
        p.H = (int)q.H; p.W = (int)q.W; p.Cin_b = (int)(q.Cin * esz); p.S = (int)q.S;
        p.PQ = (int)(q.P * q.Q); p.Q = (int)q.Q;
        p.sh = (int)q.sh; p.sw = (int)q.sw; p.ph = (int)q.ph; p.pw = (int)q.pw;
    }
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)q.batch);
    if (q.conv) hipLaunchKernelGGL((kc_kernel<INT8, T, true>), grid, dim3(T::NT), 0, q.stream, p);
    else hipLaunchKernelGGL((kc_kernel<INT8, T, false>), grid, dim3(T::NT), 0, q.stream, p);
    return hipGetLastError();
}

template <class T>
double kc_cost(const Problem &q, double eff)
{
    return tile_cost_us(q, T::BM, T::BN, T::LDS, T::NT, eff, q.in_type == XP_I8 ? 1 : 2);
}

#define XP_KC_VARIANT(NAME, TYPESTR, INT8, BM, BN, WM, WN, NS, EFF)                                            \
    bool NAME##_can(const Problem &q) { return kc_can_run_common<INT8>(q, BM, BN); }                  \
    hipError_t NAME##_launch(const Problem &q) { return kc_launch<INT8, Tile<BM, BN, WM, WN, NS>>(q); } \
    double NAME##_cost(const Problem &q) { return kc_cost<Tile<BM, BN, WM, WN, NS>>(q, EFF); }        \
    const Variant NAME = {TYPESTR " " #BM "x" #BN "x128B waves " #WM "x" #WN " stages " #NS " mfma32",  \
                          NAME##_can, NAME##_launch, NAME##_cost};

XP_KC_VARIANT(kBf256x256w2x4, "bf16", false, 256, 256, 2, 4, 2, 0.50)
XP_KC_VARIANT(kBf256x256w2x2, "bf16", false, 256, 256, 2, 2, 2, 0.45)
XP_KC_VARIANT(kBf256x128w2x2, "bf16", false, 256, 128, 2, 2, 2, 0.40)
XP_KC_VARIANT(kBf128x128w2x2, "bf16", false, 128, 128, 2, 2, 2, 0.30)
XP_KC_VARIANT(kBf64x64w2x2, "bf16", false, 64, 64, 2, 2, 2, 0.10)

XP_KC_VARIANT(kI8_256x256w2x4, "i8", true, 256, 256, 2, 4, 2, 0.50)
XP_KC_VARIANT(kI8_256x256w2x2, "i8", true, 256, 256, 2, 2, 2, 0.45)
XP_KC_VARIANT(kI8_256x128w2x2, "i8", true, 256, 128, 2, 2, 2, 0.40)
XP_KC_VARIANT(kI8_128x128w2x2, "i8", true, 128, 128, 2, 2, 2, 0.30)
XP_KC_VARIANT(kI8_64x64w2x2, "i8", true, 64, 64, 2, 2, 2, 0.10)

}  // namespace

int kc_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) {
        const Variant *v[] = {&kBf256x256w2x4, &kBf256x256w2x2, &kBf256x128w2x2, &kBf128x128w2x2, &kBf64x64w2x2};
        for (size_t i = 0; i < sizeof v / sizeof *v; ++i) out[i] = v[i];
        return (int)(sizeof v / sizeof *v);
    }
    if (in_type == XP_I8) {
        const Variant *v[] = {&kI8_256x256w2x4, &kI8_256x256w2x2, &kI8_256x128w2x2, &kI8_128x128w2x2, &kI8_64x64w2x2};
        for (size_t i = 0; i < sizeof v / sizeof *v; ++i) out[i] = v[i];
        return (int)(sizeof v / sizeof *v);
    }
    return 0;
}

}  // namespace xp
