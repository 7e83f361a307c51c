#pragma once
// (shared by xp_mfma_dl.hip, xp_mfma_dl_asm.hip and xp_mfma_dl_pair.hip, which instantiate its variants)
// MFMA kernels with direct global -> LDS loads ("dl") for operands contiguous along K:
// bf16 x bf16 -> fp32 and int8 x int8 -> int32 GEMM, strided-batched GEMM and the implicit-GEMM
// NHWC convolution (Table 5 of the paper: GEMM, Batch GEMM, Conv2D NHWC).
//
// Same tile / wave / MFMA structure as the register-staged kernels of xp_mfma_kc.hip, with a
// different Cache + Pipeline realisation (the passes of Table 4 of the paper that stage data in
// on-chip memory and overlap the copy with the computation):
//   * 16-byte buffer loads write straight into LDS (no staging registers, no LDS write
//     instructions).  One wave-level load fills 1024 contiguous LDS bytes, lane l at l*16, so
//     the chunk swizzle is applied on the source side: lane l fetches the global chunk whose
//     swizzled position is l.
//   * a ring of NS LDS buffers: the loads for K step t+NS-1 are issued at the start of step t,
//     into the buffer that was read in step t-1.  Before the one workgroup barrier of step t
//     each wave waits until its own loads for step t+1 have landed (vmcnt), which leaves the
//     loads NS-1 steps of MFMA work to complete.
//   * loads past the last K step, rows past the matrix edge and convolution taps in the zero
//     padding are redirected to an out-of-range buffer offset: the hardware writes zeros into
//     LDS and touches no memory, so the pipeline needs no conditionals.
#include "xp_internal.hpp"
#include "xp_epilogue.hpp"
#include "xp_lds_tr.hpp"

#include <cstdlib>
#include <type_traits>
#include <utility>

namespace xp {
#ifdef XP_TRACE
extern long long *g_dl_trace;             // set through xp_debug_set_dl_trace (diagnostic build only; defined in xp_mfma_dl.hip)
#endif
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr unsigned OOB = 0x80000000u;     // byte offset outside every buffer range used here

struct DlParams {
    const char *A, *B;
    char *C;
    int M, N;
    int Kb;                               // K in bytes
    int KT;                               // number of K steps
    long long lda_b, ldb_b;               // row pitches in bytes
    long long ldc;                        // elements
    long long c_plane;                    // > 0: planar output (see Problem::c_plane)
    long long strideA_b, strideB_b, strideC;
    float alpha, beta;
    int tiles_m, tiles_n, group_m;
    unsigned in_bytes;                    // convolution view
    int H, W, Cin_b, R, S, PQ, Q, sh, sw, ph, pw;
    unsigned pq_magic, q_magic;           // division by PQ and by Q as a multiplication (see fast_div)
    unsigned tap_rep;                     // conv: bit r*S set for every filter row r (a row's S mask bits times this: in every row)
    int pq_shift, q_shift;
    // two-height launches: workgroups [0, n1) tile rows [0, m_split) with the first tile type,
    // the rest tile rows [m_split, M) with the second
    int n1, m_split, tiles_m2;
#ifdef XP_TRACE
    long long *trace;                     // diagnostic build: 16 words per workgroup (shader-clock and 100 MHz time stamps)
#endif
};

template <int BM_, int BN_, int WM_, int WN_, int NS_, int RB_, bool SPREAD_ = false, int OCC_ = 1, int MF_ = 32, bool NT_ = false,
          int NSA_ = NS_, int PAIR_ = 0>
struct DlTile {
    // the two k sub-steps of a block back to back on its accumulator (see pair_loop in dl_body)
    static constexpr int PAIR = PAIR_;
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NS = NS_, RB = RB_;
    // ring depth of the A buffers (NS is that of the B buffers): one more A buffer than B buffers
    // gives the A loads an extra K step to land where LDS cannot hold a third whole stage
    static constexpr int NSA = NSA_;
    static constexpr bool ASYM = NSA_ != NS_;
    static constexpr bool NTSTORE = NT_;                 // non-temporal stores of C
    static constexpr int OCC = OCC_;                     // waves per SIMD the register budget must allow
    static constexpr bool SPREAD = SPREAD_;             // issue a step's loads a share per MFMA sub-step
    static constexpr int NWAVE = WM * WN, NT = NWAVE * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int MF = MF_;                       // MFMA block edge: 32 (32x32x16 / x32) or 16 (16x16x32 / x64)
    static constexpr int MI = WTM / MF, NI = WTN / MF;
    static constexpr int CPR = RB / 16;                 // 16-byte chunks per tile row
    static constexpr int RPI = 64 / CPR;                // tile rows filled by one wave-level load
    static constexpr int KSUB = 1024 / MF;               // bytes of K one MFMA consumes per row: 64 lanes x 16 B / MF rows
    static constexpr int PH = RB / KSUB;                 // MFMA sub-steps per K step
    // rows a K step occupies in LDS: the tile height rounded up to what one round of wave-level
    // loads fills (a tile of 208 rows is loaded as 256; rows past the tile are out of range)
    static constexpr int BMP = (BM + RPI * NWAVE - 1) / (RPI * NWAVE) * (RPI * NWAVE);
    static constexpr int BNP = (BN + RPI * NWAVE - 1) / (RPI * NWAVE) * (RPI * NWAVE);
    static constexpr int IA = BMP / RPI / NWAVE, IB = BNP / RPI / NWAVE;   // loads per wave and step
    static constexpr int A_BYTES = BMP * RB, B_BYTES = BNP * RB;   // one buffer of each ring
    static constexpr int B_BASE = NSA * A_BYTES;                   // the B ring follows the A ring
    static constexpr int LDS = NSA * A_BYTES + NS * B_BYTES;
    // loads of this wave that may still be in flight when the loads of the next K step must have landed
    static constexpr bool B_DEEP = NS_ > NSA_;           // the extra buffer goes to B (whose loads then are the ones issued last)
    static constexpr int NSMIN = NS_ < NSA_ ? NS_ : NSA_;
    static constexpr int PENDING = ASYM ? (B_DEEP ? IB : IA) + (NSMIN - 2) * (IA + IB) : (NS - 2) * (IA + IB);
    static_assert(RB == 64 || RB == 128, "row bytes");
    static_assert(MF == 32 || MF == 16, "MFMA shape");
    static_assert(WTM % MF == 0 && WTN % MF == 0, "wave sub-tile must be whole MFMA blocks");
    static_assert(PH >= 1, "a K step must hold at least one MFMA sub-step");
    static_assert(NSMIN >= 2 && NSA <= NS + 1 && NS <= NSA + 1 && PENDING + IA + IB <= 63, "ring depths; vmcnt is a 6-bit counter");
    static_assert(!ASYM || !SPREAD_, "spread issue is for equal ring depths");
    static_assert(LDS <= 160 * 1024, "LDS budget of one compute unit");
    static_assert(!SPREAD || NS >= 3, "with two buffers the loads of a step must all be issued at its start");
    static_assert(!PAIR || (NSA == 3 && NS == 2 && MF == 16 && RB == 128 && MI >= 3), "paired sub-steps: three A and two B buffers");
};

// Operand along its outer index (MODE 3-5 of dl_body): chunk swizzle of a k row of ROWB bytes.  A transposing
// read touches the 16 rows 8g + q (+4), g, q = 0..3, 32 bytes each.  Rows of 256 bytes or more all start in
// the same bank: the term, even and below 16, takes 8 different values on them (each twice: the 512 bytes of
// a read need two cycles anyway).  Rows of 128 bytes alternate between the two halves of the banks and hold
// only four 32-byte pairs: two bits, from the row bits that the alternation leaves free.
template <int ROWB> __device__ __forceinline__ int bnm_swz(int kr)
{
    static_assert(ROWB == 128 || ROWB == 256 || ROWB == 512, "bytes of one k row of the tile");
    if constexpr (ROWB == 128) return (((kr >> 1) & 1) | (((kr >> 3) & 1) << 1)) << 1;
    else return ((kr & 3) | (((kr >> 3) & 1) << 2)) << 1;
}

// Chunk swizzle: a per-row XOR of the 16-byte chunk index.  A 128-bit LDS read is served in four
// passes of 16 lanes over 64 four-byte banks; measured with SQ_LDS_BANK_CONFLICT on two-lane
// probes, a pass holds the lane quads (lane/4) of equal bit parity within one half of the wave
// (lanes 0-3, 12-15, 20-23, 24-27 form the first pass).  For each (row bytes, MFMA block size) the
// XOR term below was found by exhaustive search over XOR-linear functions of the row bits so
// that the 16 fragment reads of every pass fall into 16 different 16-byte bank groups
// (SQ_LDS_BANK_CONFLICT = 0 in the kernels).  Only row bits 0..3 are used, so the term is the
// same for every 16-row block of a tile.
template <int RB, int MF> __device__ __forceinline__ int swz(int row)
{
    if constexpr (RB == 128 && MF == 32) return (row & 7) ^ ((row >> 3) & 1);
    else if constexpr (RB == 128) return row & 6;
    else if constexpr (MF == 32) return ((row >> 1) & 3) ^ ((row >> 3) & 1);
    else return (row >> 1) & 2;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// s_waitcnt immediate for "vmcnt <= n and lgkmcnt == 0" (gfx9 encoding, expcnt left open)
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4); }

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool INT8, int MF> struct Acc;
template <> struct Acc<false, 32> {
    typedef f32x16 type;
    __device__ static __forceinline__ type mma(u32x4 a, u32x4 b, type c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                       c, 0, 0, 0);
    }
};
template <> struct Acc<true, 32> {
    typedef i32x16 type;
    __device__ static __forceinline__ type mma(u32x4 a, u32x4 b, type c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b),
                                                     c, 0, 0, 0);
    }
};
template <> struct Acc<false, 16> {
    typedef f32x4 type;
    __device__ static __forceinline__ type mma(u32x4 a, u32x4 b, type c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                       c, 0, 0, 0);
    }
};
template <> struct Acc<true, 16> {
    typedef i32x4 type;
    __device__ static __forceinline__ type mma(u32x4 a, u32x4 b, type c)
    {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b),
                                                     c, 0, 0, 0);
    }
};

// The 16x16 MFMA as assembly with its accumulator held in the accumulation registers.  A wave that owns a 128 x 128
// tile has 256 accumulator registers, the whole accumulation file; left to the register allocator, which moves values
// between the two files as it sees fit, its loop is mostly copies.
template <bool INT8> __device__ __forceinline__ void mma16_acc(typename Acc<INT8, 16>::type &c, u32x4 a, u32x4 b)
{
    if constexpr (INT8) asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// 16 bytes per lane from the accumulation registers to dst + OFFSET bytes.  The store is written through (sc0 sc1): the
// lines leave the L2 while the other stores are still being issued, instead of staying dirty until the write-back at
// the end of the kernel (4096^3 bf16: -1.4 us of 95.5; marking them non-temporal instead costs 6 us).
template <int OFFSET, typename AccT, typename OutT> __device__ __forceinline__ void store_from_acc(OutT *dst, const AccT &c)
{
    static_assert(OFFSET >= 0 && OFFSET < 4096, "the instruction's offset field");
    asm volatile("global_store_dwordx4 %0, %1, off offset:%2 sc0 sc1" : : "v"(dst), "a"(c), "n"(OFFSET) : "memory");
}

// the same from vector registers (the convolution's two tiles per compute unit: -1.5 to -2.4 us of 100); STREAM keeps
// the non-temporal stores of the variants that ask for them
template <bool STREAM, typename V4> __device__ __forceinline__ void put_tile(V4 *dst, V4 v)
{
    static_assert(sizeof(V4) == 16, "16 bytes per lane");
    if constexpr (STREAM) __builtin_nontemporal_store(v, dst);
    // (a store of more than 8 bytes reads its data a little after it is issued; the compiler keeps the next write of those
    // registers away from its own stores, for this one the wait states are spelt out: the four-wave kernels without
    // pinned accumulators copy block after block from the accumulation registers through the same four registers)
    else asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(dst), "v"(v) : "memory");
}

// Debug build (-DXP_LDS_POISON, libxp_poison.so): the 16 bytes of an LDS slot that a direct-to-LDS load is about to
// overwrite are filled with NaNs first (bf16 0x7fc0; as int8 -64 and 127), and the write has completed before the load
// is issued.  A wave that still reads the slot while the load is in flight -- a ring that is refilled too early -- then
// sees NaNs every time instead of, almost always, the old and still correct data.
__device__ __forceinline__ void lds_poison(unsigned lds_byte_address)
{
#ifdef XP_LDS_POISON
    const u32x4 nan = {0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u};
    asm volatile("ds_write_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : : "v"(lds_byte_address), "v"(nan) : "memory");
#else
    (void)lds_byte_address;
#endif
}

// floor(n / d) for 0 <= n < 2^31 as a multiplication: magic = ceil(2^(31 + shift) / d) with shift = ceil(log2 d)
// (the host works both out once per call); exact for every such n.  A 32-bit division costs some forty vector
// instructions, and the convolution's set-up has two per load slot.
__device__ __forceinline__ int fast_div(int n, unsigned magic, int shift)
{
    return (int)(((unsigned long long)(unsigned)n * magic) >> (31 + shift));
}

// One tile of C.  `bid` numbers the tiles of the row range [m_base, m_end) of the problem, which is
// tiles_m tile-rows high; lds points at T::LDS bytes of shared memory.
// MODE: 0 GEMM, 1 convolution (A addressed through the im2col map), 2 convolution with planar output
// (a kernel of its own, so that the epilogue branch costs the others nothing: with the branch in
// every kernel the NHWC convolution lost 2.4 %)
template <bool INT8, class T, int MODE>
__device__ __forceinline__ void dl_body(const DlParams &p, char *lds, int bid, int m_base, int m_end, int tiles_m)
{
    constexpr bool CONV = MODE == 1 || MODE == 2 || MODE == 7 || MODE == 8, PLANAR = MODE == 2 || MODE == 8;
    // MODE 3: GEMM whose B is contiguous along N (row-major B, the usual layout of a framework's weights
    // and activations).  Its tile lies in LDS as it lies in memory -- one k per row of BN columns, filled
    // by the same direct-to-LDS loads -- and a fragment (8 consecutive k of one column) is gathered by the
    // transposing LDS read (ds_read_b64_tr_b16: in a block of 16 lanes, lane i receives as value j the
    // element i&3 of the 8 bytes addressed by lane 4j + (i>>2)); two of them per fragment.
    // MODE 4: the same for A contiguous along M (a column-major A); MODE 5: both.  ASMR: one of them, all
    // fragment reads are assembly.
    // MODE 6, 7, 8: MODE 0, 1, 2 with their (plain) fragment reads as assembly too, which buys the main loop
    // in rounds with constant ring positions (below).
    constexpr bool BNM = MODE == 3 || MODE == 5, AMM = MODE == 4 || MODE == 5, ASMR = MODE >= 3;
    static_assert(!ASMR || (T::MF == 16 && T::RB == 128), "assembly reads: 16x16 blocks, 128 bytes of K per step");
    static_assert(!(AMM || BNM) || !INT8, "operand along its outer index: bf16");
    constexpr int RBN = T::BN * 2;                        // BNM: bytes of one k row of the B tile
    constexpr int RAM = T::BM * 2;                        // AMM: bytes of one k row of the A tile
    using AccT = typename Acc<INT8, T::MF>::type;
    constexpr int RB = T::RB, MF = T::MF;
    constexpr int NACC = MF == 32 ? 16 : 4;           // accumulator registers per lane and block

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / T::WN, wn = wave % T::WN;
#ifdef XP_TRACE
    // diagnostic build (-DXP_TRACE): where a workgroup's time goes -- entry, first MFMA, end of the K loop, stores done
    long long tr_c[4] = {0, 0, 0, 0}, tr_w[4] = {0, 0, 0, 0};
    long long tr_wait[3] = {0, 0, 0};                   // paired loop, wave 0: cycles waiting for global loads, in the barrier, and from entry to the first load
    const int tr_slot = (int)(blockIdx.y * gridDim.x + blockIdx.x) + (m_base ? (int)(gridDim.x * gridDim.y) : 0);
    tr_c[0] = clock64(); tr_w[0] = wall_clock64();
#endif

    // workgroup -> tile: one XCD (workgroup id mod 8) owns a run of consecutive tiles, walked in
    // groups of group_m tile-rows, so that the tiles sharing an L2 share A and B panels
    const int nb = tiles_m * p.tiles_n;
    long long batch = blockIdx.y;
    if (gridDim.y > 1 && m_base == 0 && m_end == p.M && (nb < 64 || (nb & 7) != 0)) {
        // batched problems of a few tiles each (one tile height per launch): the tiles of a problem would be
        // dealt to different XCDs and each L2 would fetch the problem's operands again (with 8 tiles a problem,
        // tile x of every problem would run on XCD x: the shared operand fetched 8 times)
        unsigned x, y;
        xcd_batch_remap(x, y);
        bid = (int)x;
        batch = y;
    } else if ((nb & 7) == 0) {
        bid = (bid & 7) * (nb >> 3) + (bid >> 3);
    }
    const int gsz = p.group_m * p.tiles_n;
    const int g = bid / gsz, first_m = g * p.group_m;
    const int gm = min(tiles_m - first_m, p.group_m);
    const int tm = first_m + (bid % gsz) % gm, tn = (bid % gsz) / gm;
    const int m0 = m_base + tm * T::BM, n0 = tn * T::BN;

    const int rows_a = min(m_end - m0, T::BM), rows_b = min(p.N - n0, T::BN);
    __amdgpu_buffer_rsrc_t ra, rb;
    // Convolution: a lane's offset for a filter tap is its pixel's offset (fixed) plus the tap's offset
    // (the same for every lane: a scalar), so the loop only has to decide whether the tap falls inside
    // the image for that pixel -- one bit of a mask worked out here, once.  Pixel offsets are taken
    // relative to (-pad_h, -pad_w) so that they are never negative; the buffer starts that much earlier.
    const int conv_bias = CONV ? (p.ph * p.W + p.pw) * p.Cin_b : 0;
    if constexpr (CONV) {
        ra = make_rsrc(p.A - conv_bias, p.in_bytes + (unsigned)conv_bias);
    } else if constexpr (AMM) {                           // lda_b: bytes from one k row to the next
        ra = make_rsrc(p.A + batch * p.strideA_b + (long long)m0 * 2, (unsigned)((long long)(p.Kb / 2 - 1) * p.lda_b + (long long)rows_a * 2));
    } else {
        ra = make_rsrc(p.A + batch * p.strideA_b + (long long)m0 * p.lda_b,
                       (unsigned)((long long)(rows_a - 1) * p.lda_b + p.Kb));
    }
    if constexpr (BNM)                                    // ldb_b: bytes from one k row to the next
        rb = make_rsrc(p.B + batch * p.strideB_b + (long long)n0 * 2, (unsigned)((long long)(p.Kb / 2 - 1) * p.ldb_b + (long long)rows_b * 2));
    else
        rb = make_rsrc(p.B + batch * p.strideB_b + (long long)n0 * p.ldb_b,
                       (unsigned)((long long)(rows_b - 1) * p.ldb_b + p.Kb));

    // load slots: slot i of this wave fills the 1024 LDS bytes of row block (wave + i*NWAVE);
    // lane l lands at row l/CPR, position l%CPR, and fetches the chunk that belongs there
    unsigned a_off_g[T::IA], b_off_g[T::IB];            // byte offsets of this lane's chunks in global memory
    // Byte offset of the fetched chunk within the row, for the end-of-K test: a_cb0 + i * A_CB_STEP for load i.
    // Along K the offset is the same for every load of the lane (a wave's loads are a multiple of 16 rows apart
    // and the swizzle uses row bits 0..3 only); along the outer index the loads are whole k rows apart.
    static_assert((T::NWAVE * T::RPI) % 16 == 0, "the loads of a lane differ in row bits above the swizzle's");
    constexpr int A_CB_STEP = AMM ? 2 * T::NWAVE * (1024 / RAM) : 0, B_CB_STEP = BNM ? 2 * T::NWAVE * (1024 / RBN) : 0;
    int a_cb0 = 0, b_cb0 = 0;
    int a_outside[CONV ? T::IA : 1];                    // conv: bit r*S + s set <=> tap (r, s) of this lane's pixel is padding
#pragma unroll
    for (int i = 0; i < T::IA; ++i) {
        const int row = (wave + i * T::NWAVE) * T::RPI + lane / T::CPR;
        const int a_cb = ((lane % T::CPR) ^ swz<RB, T::MF>(row)) << 4;
        if (i == 0) a_cb0 = a_cb;
        if constexpr (AMM) {                            // as for B along N below
            const int kr = (wave + i * T::NWAVE) * (1024 / RAM) + lane / (RAM / 16);
            const int chunk = (lane % (RAM / 16)) ^ bnm_swz<RAM>(kr);
            if (i == 0) a_cb0 = kr * 2;
            a_off_g[i] = m0 + chunk * 8 < m_end ? (unsigned)(kr * p.lda_b) + (chunk << 4) : OOB;
        } else if constexpr (CONV) {
            const int m = m0 + row;
            a_outside[i] = -1;                          // a row past the end: every tap is outside
            a_off_g[i] = 0;
            if (m < m_end && row < T::BM) {
                const int n = fast_div(m, p.pq_magic, p.pq_shift), pq = m - n * p.PQ;
                const int op = fast_div(pq, p.q_magic, p.q_shift), oq = pq - op * p.Q;
                const int h0 = op * p.sh - p.ph, w0 = oq * p.sw - p.pw;
                a_off_g[i] = (unsigned)n * (unsigned)(p.H * p.W) * (unsigned)p.Cin_b +
                             (unsigned)((h0 + p.ph) * p.W + w0 + p.pw) * (unsigned)p.Cin_b + a_cb;
                // Without loops (a wave issues one instruction every few cycles and nothing else runs on its SIMD: the
                // set-up's instruction count is the time before the first load).  Columns s of the window inside the
                // image: [max(-w0, 0), min(W - w0, S)); rows likewise; a row outside the image is outside with all
                // its columns, the others share the columns' bits (their S bits times tap_rep: in every row)
                auto low_bits = [](int n) { return n >= 32 ? 0xffffffffu : (1u << n) - 1u; };     // 0 <= n
                const int c_lo = min(max(-w0, 0), p.S), c_hi = min(max(p.W - w0, 0), p.S);
                const int r_lo = min(max(-h0, 0), p.R), r_hi = min(max(p.H - h0, 0), p.R);
                const unsigned cols_out = low_bits(c_lo) | (low_bits(p.S) & ~low_bits(c_hi));
                const unsigned rows_in = r_hi > r_lo ? low_bits(r_hi * p.S) & ~low_bits(r_lo * p.S) : 0u;
                a_outside[i] = (int)((low_bits(p.R * p.S) & ~rows_in) | ((cols_out * p.tap_rep) & rows_in));
            }
        } else {
            a_off_g[i] = (unsigned)(row * p.lda_b) + a_cb;
        }
    }
#pragma unroll
    for (int i = 0; i < T::IB; ++i) {
        if constexpr (BNM) {
            // a wave-level load fills 1024 LDS bytes = 1024 / RBN k rows; the lane at chunk position pc of
            // k row kr fetches chunk pc ^ swizzle(kr) of that row (a chunk: 8 columns)
            const int kr = (wave + i * T::NWAVE) * (1024 / RBN) + lane / (RBN / 16);
            const int chunk = (lane % (RBN / 16)) ^ bnm_swz<RBN>(kr);
            if (i == 0) b_cb0 = kr * 2;                    // so that the end-of-K test (kb + b_cb >= Kb) means k >= K
            b_off_g[i] = n0 + chunk * 8 < p.N ? (unsigned)(kr * p.ldb_b) + (chunk << 4) : OOB;
        } else {
            const int row = (wave + i * T::NWAVE) * T::RPI + lane / T::CPR;
            const int b_cb = ((lane % T::CPR) ^ swz<RB, T::MF>(row)) << 4;
            if (i == 0) b_cb0 = b_cb;
            b_off_g[i] = (unsigned)(row * p.ldb_b) + b_cb;
        }
    }
    // BNM fragment reads: lane a = l%16 of block g = l/16 addresses k row 8g + (a >> 2) (+ 32 per sub-step,
    // + 4 for the second read), the 8 bytes at columns 16j + 4*(a & 3) of the wave's column range
    const unsigned lds_base = lds_address(lds);
    int fbn[BNM ? T::NI : 1];
    if constexpr (BNM) {
        const int a16 = lane & 15, kr = 8 * (lane >> 4) + (a16 >> 2);
#pragma unroll
        for (int j = 0; j < T::NI; ++j) {
            const int chunk = (wn * T::WTN + 16 * j) / 8 + ((a16 & 3) >> 1);
            fbn[j] = kr * RBN + ((chunk ^ bnm_swz<RBN>(kr)) << 4) + 8 * (a16 & 1);
        }
    }

    int fam[AMM ? T::MI : 1];
    if constexpr (AMM) {
        const int a16 = lane & 15, kr = 8 * (lane >> 4) + (a16 >> 2);
#pragma unroll
        for (int i = 0; i < T::MI; ++i) {
            const int chunk = (wm * T::WTM + 16 * i) / 8 + ((a16 & 3) >> 1);
            fam[i] = kr * RAM + ((chunk ^ bnm_swz<RAM>(kr)) << 4) + 8 * (a16 & 1);
        }
    }

    // fragment reads: lane l reads row l % MF of an MF-row block, chunk (64/MF)*kk + l / MF
    const int frow = lane & (MF - 1), fch = lane / MF;
    const int fsw = swz<RB, T::MF>(frow);                      // blocks start at multiples of 16 rows
    int fa[T::PH], fb[T::PH];
#pragma unroll
    for (int kk = 0; kk < T::PH; ++kk) {
        const int c = (((64 / MF) * kk + fch) ^ fsw) << 4;
        fa[kk] = (wm * T::WTM + frow) * RB + c;
        fb[kk] = (wn * T::WTN + frow) * RB + c;
    }

    AccT acc[T::MI][T::NI];
#pragma unroll
    for (int i = 0; i < T::MI; ++i)
#pragma unroll
        for (int j = 0; j < T::NI; ++j)
#pragma unroll
            for (int v = 0; v < NACC; ++v) acc[i][j][v] = 0;

    int tap_s = 0, tap = 0, tap_off = 0, c0_b = 0;      // conv: filter tap and channel offset of the next step to load
    const int roll_step = CONV ? (p.W - p.S) * p.Cin_b : 0;

    // issue A loads [lo, hi) of K step kt into the A buffer at byte offset a_off; likewise for B
    constexpr int IT = T::IA + T::IB;
    // CHECK: the step may reach or pass the end of K, so every lane tests its chunk; the main part of
    // the loop issues whole steps only and spends no vector instruction on that (matrix and vector
    // instructions do not overlap on a SIMD: vector work in the loop is MFMA time lost)
    auto issue_a = [&](int kt, int a_off, int lo, int hi, auto check_c) {
        constexpr bool CHECK = decltype(check_c)::value;
        const int kb = kt * RB;
#pragma unroll
        for (int i = 0; i < T::IA; ++i) {
            if (i < lo || i >= hi) continue;
            unsigned off;
            int soff;
            if constexpr (CONV) {
                // bit `tap` of the mask, spread over the word, puts a padding tap beyond the buffer's range
                off = ((unsigned)__builtin_amdgcn_sbfe(a_outside[i], tap, 1) & OOB) | a_off_g[i];
                soff = c0_b + tap_off;
            } else {
                off = a_off_g[i];
                soff = AMM ? (int)((unsigned)kt * (RB / 2) * (unsigned)p.lda_b) : kb;
            }
            if constexpr (CHECK) {
                if (kb + a_cb0 + i * A_CB_STEP >= p.Kb) off = OOB;
            }
            lds_void *dst = (lds_void *)(lds + a_off + (wave + i * T::NWAVE) * 1024);
            lds_poison(lds_base + a_off + (wave + i * T::NWAVE) * 1024 + lane * 16);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, dst, 16, off, soff, 0, 0);
        }
        if constexpr (CONV) {
            if (hi >= T::IA && lo < T::IA) {            // the step's A loads are all issued: advance (tap, channel offset)
                // (arithmetic on 0 / -1 masks, neither selects nor branches: the compiler turns selects into branches
                // here, which cuts the unrolled rounds into pieces and costs it some thirty registers)
                c0_b += RB;
                const int wrap = (p.Cin_b - 1 - c0_b) >> 31;             // -1 when the channels of the tap are used up
                c0_b &= ~wrap;
                tap -= wrap;
                tap_s -= wrap;
                const int roll = (p.S - 1 - tap_s) >> 31;                // -1 when the tap row is used up
                tap_s &= ~roll;
                tap_off += (p.Cin_b & wrap) + (roll_step & roll);          // next tap: one pixel on; next tap row: W - S more
            }
        }
    };
    auto issue_b = [&](int kt, int b_off, int lo, int hi, auto check_c) {
        constexpr bool CHECK = decltype(check_c)::value;
        const int kb = kt * RB;
#pragma unroll
        for (int i = 0; i < T::IB; ++i) {
            if (i < lo || i >= hi) continue;
            unsigned off = b_off_g[i];
            if constexpr (CHECK) {
                if (kb + b_cb0 + i * B_CB_STEP >= p.Kb) off = OOB;
            }
            lds_void *dst = (lds_void *)(lds + b_off + (wave + i * T::NWAVE) * 1024);
            lds_poison(lds_base + b_off + (wave + i * T::NWAVE) * 1024 + lane * 16);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, dst, 16, off, BNM ? (int)((unsigned)kt * (RB / 2) * (unsigned)p.ldb_b) : kb, 0, 0);
        }
    };
    // loads [lo, hi) of the IA + IB that one K step issues when both rings have the same depth
    auto issue = [&](int kt, int a_off, int b_off, int lo, int hi, auto check_c) {
        issue_a(kt, a_off, lo, hi < T::IA ? hi : T::IA, check_c);
        issue_b(kt, b_off, lo > T::IA ? lo - T::IA : 0, hi - T::IA, check_c);
    };
    // ASMR: every fragment read is assembly (see xp_lds_tr.hpp): offsets are instruction constants, the waits are
    // explicit.  AO / BO: byte offsets of the A / B buffer as constants (the unrolled main loop), or -1: taken from
    // a_off / b_off at run time (one vector addition per address register).  An offset field holds 16 bits;
    // buffers further up are reached from a second set of address registers 64 KB higher.
    constexpr int A_TOP = AMM ? 36 * RAM : (T::MI - 1) * MF * RB;        // largest offset within a buffer
    constexpr int B_TOP = BNM ? 36 * RBN : (T::NI - 1) * MF * RB;
    constexpr int NFA = AMM ? T::MI : T::PH, NFB = BNM ? T::NI : T::PH;  // address registers per operand
    constexpr bool A_FAR = ASMR && (T::NSA - 1) * T::A_BYTES + A_TOP >= 65536;
    constexpr bool B_FAR = ASMR && (T::NS - 1) * T::B_BYTES + B_TOP >= 65536;
    unsigned fa_far[A_FAR ? NFA : 1], fb_far[B_FAR ? NFB : 1];
    if constexpr (A_FAR)
        for (int x = 0; x < NFA; ++x) fa_far[x] = lds_base + (AMM ? fam[AMM ? x : 0] : fa[AMM ? 0 : x]) + 65536;
    if constexpr (B_FAR)
        for (int x = 0; x < NFB; ++x) fb_far[x] = lds_base + T::B_BASE + (BNM ? fbn[BNM ? x : 0] : fb[BNM ? 0 : x]) + 65536;
    // A fragment as the reads deliver it: one 16-byte read, or the two 8-byte halves of a pair of transposing reads.
    // The halves stay separate values until the wait for them has passed (frag_tie); composing the four words
    // earlier would let a register copy run ahead of the data.
    using AFrag = typename std::conditional<AMM, FragHalves, u32x4>::type;
    using BFrag = typename std::conditional<BNM, FragHalves, u32x4>::type;
    // one fragment of the set: F < NI the B fragment F, else the A fragment F - NI (the B fragments first: every
    // block row of the next sub-step needs all of them).  Operand along K: one address register per sub-step, the
    // blocks are offsets; operand along its outer index: one address register per block (the swizzle), the sub-step
    // is an offset
    // (each read picks the near or the far address register by its own constant offset: a buffer may straddle 64 KB)
    auto read_a_asm = [&](auto ao_c, auto kk_c, auto i_c, int a_off, AFrag &dst) {
        constexpr int AO = decltype(ao_c)::value, KK = decltype(kk_c)::value, I = decltype(i_c)::value;
        constexpr int AREL = AO < 0 ? 0 : AO;
        if constexpr (AMM) {
            constexpr int LO = AREL + KK * 32 * RAM, HI = LO + 4 * RAM;
            constexpr bool FAR_LO = LO >= 65536, FAR_HI = HI >= 65536;
            const unsigned near = AO < 0 ? lds_base + a_off + fam[I] : lds_base + fam[I];
            const unsigned far = fa_far[A_FAR ? I : 0];
            dst.lo = lds_read_tr16_b64<FAR_LO ? LO - 65536 : LO>(FAR_LO ? far : near);
            dst.hi = lds_read_tr16_b64<FAR_HI ? HI - 65536 : HI>(FAR_HI ? far : near);
        } else {
            constexpr int OFFS = AREL + I * MF * RB;
            constexpr bool FAR = OFFS >= 65536;
            const unsigned at = AO < 0 ? lds_base + a_off + fa[KK] : (FAR ? fa_far[A_FAR ? KK : 0] : lds_base + fa[KK]);
            dst = lds_read_b128<FAR ? OFFS - 65536 : OFFS>(at);
        }
    };
    auto read_b_asm = [&](auto bo_c, auto kk_c, auto j_c, int b_off, BFrag &dst) {
        constexpr int BO = decltype(bo_c)::value, KK = decltype(kk_c)::value, J = decltype(j_c)::value;
        constexpr int BREL = BO < 0 ? 0 : BO - T::B_BASE;
        const unsigned b_rt = lds_base + b_off;          // used with a run-time buffer offset only
        if constexpr (BNM) {
            constexpr int LO = BREL + KK * 32 * RBN, HI = LO + 4 * RBN;
            constexpr bool FAR_LO = LO >= 65536, FAR_HI = HI >= 65536;
            const unsigned near = BO < 0 ? b_rt + fbn[J] : lds_base + T::B_BASE + fbn[J];
            const unsigned far = fb_far[B_FAR ? J : 0];
            dst.lo = lds_read_tr16_b64<FAR_LO ? LO - 65536 : LO>(FAR_LO ? far : near);
            dst.hi = lds_read_tr16_b64<FAR_HI ? HI - 65536 : HI>(FAR_HI ? far : near);
        } else {
            constexpr int OFFS = BREL + J * MF * RB;
            constexpr bool FAR = OFFS >= 65536;
            const unsigned at = BO < 0 ? b_rt + fb[KK] : (FAR ? fb_far[B_FAR ? KK : 0] : lds_base + T::B_BASE + fb[KK]);
            dst = lds_read_b128<FAR ? OFFS - 65536 : OFFS>(at);
        }
    };
    auto read_frag_asm = [&](auto ao_c, auto bo_c, auto kk_c, auto f_c, int a_off, int b_off, AFrag (&af)[T::MI], BFrag (&bf)[T::NI]) {
        constexpr int F = decltype(f_c)::value;
        if constexpr (F >= T::NI) read_a_asm(ao_c, kk_c, std::integral_constant<int, F - T::NI>{}, a_off, af[F - T::NI]);
        else read_b_asm(bo_c, kk_c, f_c, b_off, bf[F]);
    };
    // One MFMA sub-step on the set (ca, cb) with the reads of the set (na, nb) -- sub-step KK of the buffers at
    // AO / BO -- dealt out behind its block rows: a wave that issues its reads as one burst keeps the matrix pipe
    // idle meanwhile when its SIMD neighbour, in step with it, does the same (a cycle counter in the kernel shows
    // 2430 cycles per K step with bursts, 2140 dealt out; 2048 is the MFMA time).  The last block rows get no reads, so
    // that the reads have returned when the step's barrier asks for it.  Columns are walked back and forth: between
    // two consecutive MFMAs only one operand changes.  after_row(i) is called behind block row i (the second sub-step
    // of a K step issues the step's global loads there, a share per row).  Every wait is for all LDS operations of the
    // wave (the counter also counts scalar loads, which may return out of order: no partial waits).
    auto weave = [&](auto ao_c, auto bo_c, auto kk_c, int a_off, int b_off, AFrag (&ca)[T::MI], BFrag (&cb)[T::NI], AFrag (&na)[T::MI],
                     BFrag (&nb)[T::NI], auto &&after_row) {
        constexpr int NF = T::MI + T::NI;                               // fragments to read
        constexpr int ROWS = T::MI > 2 ? T::MI - 2 : 1;                 // block rows that carry reads
        constexpr int PER = (NF + ROWS - 1) / ROWS;
        lds_wait<0>();                                                  // (ca, cb) were read during the sub-step before
#pragma unroll
        for (int i = 0; i < T::MI; ++i) frag_tie(ca[i]);
#pragma unroll
        for (int j = 0; j < T::NI; ++j) frag_tie(cb[j]);
        static_for<T::MI>([&](auto i_c) {
            constexpr int I = decltype(i_c)::value;
#pragma unroll
            for (int jj = 0; jj < T::NI; ++jj) {
                const int j = (I & 1) ? T::NI - 1 - jj : jj;
                // 16x16 blocks are computed transposed (B fragment as the first operand): see mma_all
                if constexpr (MF == 16) acc[I][j] = Acc<INT8, 16>::mma(frag_value(cb[j]), frag_value(ca[I]), acc[I][j]);
            }
            __builtin_amdgcn_sched_barrier(0);
            static_for<PER>([&](auto r_c) {
                constexpr int F = I * PER + decltype(r_c)::value;
                if constexpr (F < NF) read_frag_asm(ao_c, bo_c, kk_c, std::integral_constant<int, F>{}, a_off, b_off, na, nb);
            });
            after_row(i_c);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto read_frags = [&](int a_off, int b_off, int kk, u32x4 (&af)[T::MI], u32x4 (&bf)[T::NI]) {
#pragma unroll
        for (int i = 0; i < T::MI; ++i) af[i] = *(const u32x4 *)(lds + a_off + fa[kk] + i * MF * RB);
#pragma unroll
        for (int j = 0; j < T::NI; ++j) bf[j] = *(const u32x4 *)(lds + b_off + fb[kk] + j * MF * RB);
    };
    auto mma_all = [&](u32x4 (&af)[T::MI], u32x4 (&bf)[T::NI]) {
#pragma unroll
        for (int i = 0; i < T::MI; ++i)
#pragma unroll
            for (int j = 0; j < T::NI; ++j) {
                // 16x16 blocks are computed transposed (B fragment as the first operand) so that a
                // lane ends up with 4 consecutive columns of C: one 16-byte store per block
                if constexpr (MF == 32) acc[i][j] = Acc<INT8, 32>::mma(af[i], bf[j], acc[i][j]);
                else acc[i][j] = Acc<INT8, 16>::mma(bf[j], af[i], acc[i][j]);
            }
    };

    const int KT = p.KT;
    constexpr int PENDING = T::PENDING;                  // loads that may still be in flight at a barrier
    constexpr int A_END = T::NSA * T::A_BYTES, B_END = T::B_BASE + T::NS * T::B_BYTES;
    if constexpr (T::PAIR != 0) {
        // Paired sub-steps.  Two MFMAs in a row on the same accumulator draw less power than the same two with other
        // blocks between them (a loop of nothing but MFMAs on N(0,1) operands at the power limit: 2180 against 2040
        // TFLOP/s; chains of four are no better, and walking the sub-steps back and forth is not either), and power is
        // what bounds this loop.  So a block takes both k sub-steps of a K step at once, which needs both sub-steps'
        // fragments of its row and column in registers: all of the step's B fragments are held (2 NI of them) and A
        // streams through four sets of two fragments, a set per block row, in groups of two rows.  Behind the first
        // row of a group go the reads for the next group and the second row covers their latency; every wait is for
        // all LDS operations.
        //   groups 0 .. MI/2-2 | barrier | group MI/2-1
        // The one barrier of step kt precedes its last group: behind it K step kt+1 is in LDS for every wave -- the last
        // group reads all of its B fragments and its first two A rows -- and every wave has finished with the buffers
        // of step kt.  The B buffer is refilled at once, by the last group, with step kt+2, which must have landed at
        // the next barrier; the A buffer by the groups before the next barrier, with step kt+3: those loads are the
        // youngest at that barrier and stay in flight across it (three A buffers, two B buffers).
        static_assert(ASMR && T::PH == 2, "paired sub-steps: with assembly reads");
        typedef std::integral_constant<int, -1> RunTime;
        typedef std::integral_constant<int, 0> Zero;
        // Block rows are counted from OFF: an odd number of rows gets a row 0 that does not exist, so that the groups
        // stay pairs and the last group, which carries the most reads, has both its rows.  Row v uses fragment set
        // v % 4; when the (even) row count is no multiple of four the sets of odd K steps are the other two.
        constexpr int OFF = T::MI & 1, MV = T::MI + OFF;
        constexpr bool ROT = MV % 4 == 2;
        constexpr int NG = MV / 2;                                      // groups of two block rows
        constexpr int NBF = 2 * T::NI;                                  // B fragments of a step
        constexpr int LAST = NG - 1;                                    // the group behind the barrier
        constexpr bool ACC_FILE = T::NWAVE == 4;                        // one wave per SIMD: accumulators in the accumulation registers
        static_assert(NG >= 2, "at least three block rows");
        if (KT > 0) {
            AFrag ar[4][2];                                             // fragment sets: sub-steps 0 and 1 of a block row
            BFrag bx[2][T::NI], by[2][T::NI];                           // the B fragments of even / odd K steps
#ifdef XP_TRACE
            tr_wait[2] = clock64() - tr_c[0];                           // (set-up: entry to the first load)
#endif
            issue_a(0, 0, 0, T::IA, std::true_type{});
            issue_b(0, T::B_BASE, 0, T::IB, std::true_type{});
            issue_a(1, T::A_BYTES, 0, T::IA, std::true_type{});
            issue_b(1, T::B_BASE + T::B_BYTES, 0, T::IB, std::true_type{});
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(IT));           // K step 0 has landed
            __builtin_amdgcn_s_barrier();
            static_for<NBF>([&](auto f_c) {
                constexpr int F = decltype(f_c)::value;
                read_b_asm(std::integral_constant<int, T::B_BASE>{}, std::integral_constant<int, F / T::NI>{},
                           std::integral_constant<int, F % T::NI>{}, 0, bx[F / T::NI][F % T::NI]);
            });
            static_for<4>([&](auto f_c) {
                constexpr int F = decltype(f_c)::value, V = F / 2;
                if constexpr (V >= OFF) read_a_asm(Zero{}, std::integral_constant<int, F % 2>{}, std::integral_constant<int, V - OFF>{}, 0, ar[V][F % 2]);
            });
            // ring state of the run-time steps: the A buffers of steps kt, kt+1, kt+2 and the B buffers of kt+1, kt (= kt+2)
            int cur_a = 0, nxt_a = T::A_BYTES, fill_a = 2 * T::A_BYTES, nxt_b = T::B_BASE + T::B_BYTES, fill_b = T::B_BASE;
            // The last K step of a tile that the whole-tile epilogue will store as it is (one wave per SIMD): a block
            // row is final when the step has passed it, so its stores go out behind the MFMAs of the row after it, one
            // behind each pair -- all but the last row's output is on its way when the loop ends.  That step issues no
            // load and reads nothing of a next step, so it needs no barrier either.
            using OutT = typename std::conditional<INT8, int, float>::type;
            constexpr bool EARLY = ACC_FILE && MF == 16 && !PLANAR && !T::NTSTORE;
            OutT *early = nullptr;                                      // where the block row that is stored next begins
            long long early_step = 0;
            if constexpr (EARLY) {
                OutT *C = (OutT *)p.C + batch * p.strideC;
                if (m0 + T::BM <= m_end && n0 + T::BN <= p.N && (INT8 || (p.beta == 0.0f && p.alpha == 1.0f)) &&
                    (((unsigned long long)C | (unsigned long long)(p.ldc * (long long)sizeof(OutT))) & 15) == 0) {
                    early = C + (long long)(m0 + wm * T::WTM + (lane & 15)) * p.ldc + (n0 + wn * T::WTN + (lane >> 4) * 4);
                    early_step = 16 * p.ldc;
                }
            }
            auto step = [&](int kt, auto odd_c, auto check_c, auto pos_c, auto final_c) {
                constexpr bool ODD = decltype(odd_c)::value;
                constexpr bool FINAL = decltype(final_c)::value;
                constexpr int POS = decltype(pos_c)::value;
                constexpr int CA = POS < 0 ? -1 : (POS % 3) * T::A_BYTES, NA = POS < 0 ? -1 : ((POS + 1) % 3) * T::A_BYTES;
                constexpr int NB = POS < 0 ? -1 : T::B_BASE + ((POS + 1) % 2) * T::B_BYTES;
                const int now_a = POS >= 0 ? CA : cur_a, next_a = POS >= 0 ? NA : nxt_a, next_b = POS >= 0 ? NB : nxt_b;
                const int into_a = POS >= 0 ? ((POS + 2) % 3) * T::A_BYTES : fill_a;
                const int into_b = POS >= 0 ? T::B_BASE + (POS % 2) * T::B_BYTES : fill_b;
                constexpr int SO = ROT && ODD ? 2 : 0, SN = ROT && !ODD ? 2 : 0;    // set offsets of this step's rows and of the next step's
                BFrag (&bc)[2][T::NI] = ODD ? by : bx;
                BFrag (&bn)[2][T::NI] = ODD ? bx : by;
                static_for<NG>([&](auto g_c) {
                    constexpr int G = decltype(g_c)::value, R0 = 2 * G, R1 = 2 * G + 1;     // (counted from OFF)
                    constexpr bool REAL0 = R0 >= OFF;
                    if constexpr (G != LAST || FINAL) lds_wait<0>();    // (the last group follows the barrier's wait)
                    if constexpr (G == 0) {
#pragma unroll
                        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                            for (int j = 0; j < T::NI; ++j) frag_tie(bc[kk][j]);
                    }
                    if constexpr (REAL0) { frag_tie(ar[(R0 + SO) % 4][0]); frag_tie(ar[(R0 + SO) % 4][1]); }
                    frag_tie(ar[(R1 + SO) % 4][0]); frag_tie(ar[(R1 + SO) % 4][1]);
                    // What the group issues besides its MFMAs, in this order: the four A fragments of the next group's
                    // rows (of this K step, or the first two rows of the next one); the last group: the next step's B
                    // fragments and the B loads of step kt+2; the others: their share of the A loads of step kt+2
                    // (into the buffer that the barrier of the step before has freed)
                    constexpr int NRB = G == LAST ? NBF : 0;
                    constexpr int L_LO = G == LAST ? 0 : G * T::IA / LAST, L_HI = G == LAST ? T::IB : (G + 1) * T::IA / LAST;
                    constexpr int NITEMS = 4 + NRB + (L_HI - L_LO);
                    auto item = [&](auto k_c) {
                        constexpr int K = decltype(k_c)::value;
                        if constexpr (K < 4) {
                            constexpr int RN = R0 + 2 + K / 2, KK = K % 2;
                            if constexpr (RN < MV)
                                read_a_asm(std::integral_constant<int, CA>{}, std::integral_constant<int, KK>{}, std::integral_constant<int, RN - OFF>{}, now_a,
                                           ar[(RN + SO) % 4][KK]);
                            else if constexpr (FINAL)
                                ;
                            else if constexpr (RN - MV >= OFF)
                                read_a_asm(std::integral_constant<int, NA>{}, std::integral_constant<int, KK>{}, std::integral_constant<int, RN - MV - OFF>{},
                                           next_a, ar[(RN - MV + SN) % 4][KK]);
                        } else if constexpr (FINAL) {
                            ;
                        } else if constexpr (K < 4 + NRB) {
                            constexpr int F = K - 4;
                            read_b_asm(std::integral_constant<int, NB>{}, std::integral_constant<int, F / T::NI>{},
                                       std::integral_constant<int, F % T::NI>{}, next_b, bn[F / T::NI][F % T::NI]);
                        } else if constexpr (K < NITEMS) {
                            constexpr int L = L_LO + K - 4 - NRB;
                            if constexpr (G == LAST) issue_b(kt + 2, into_b, L, L + 1, check_c);
                            else issue_a(kt + 2, into_a, L, L + 1, check_c);
                        }
                    };
                    // One wave per SIMD: an item behind every MFMA, so that the matrix pipe never waits for the wave to
                    // get through a run of other instructions (nobody else issues on this SIMD).  Two waves per SIMD:
                    // the reads behind the first row (the second covers their latency), the loads split over both rows.
                    constexpr int PER_ROW = 2 * T::NI;                                          // MFMAs of a block row
                    constexpr int SLOTS = (REAL0 ? 2 : 1) * PER_ROW;
                    static_assert(!ACC_FILE || (4 + NRB <= SLOTS - 8 && NITEMS <= SLOTS), "the last MFMAs of a group cover the reads' latency");
                    // (one wave per SIMD) what follows MFMA number S of the group: the reads one behind each of the
                    // first MFMAs; the loads behind every second MFMA where the group has room for that
                    constexpr int LSTEP = 4 + NRB + 2 * (L_HI - L_LO) <= SLOTS ? 2 : 1;
                    auto slot = [&](auto s_c) {
                        constexpr int S = decltype(s_c)::value;
                        if constexpr (S < 4 + NRB) item(s_c);
                        else if constexpr ((S - 4 - NRB) % LSTEP == 0) item(std::integral_constant<int, 4 + NRB + (S - 4 - NRB) / LSTEP>{});
                    };
                    auto row = [&](auto r_c, auto first_c) {
                        constexpr int I = decltype(r_c)::value - OFF, S = (decltype(r_c)::value + SO) % 4, FIRST = decltype(first_c)::value;
                        static_for<T::NI>([&](auto jj_c) {
                            constexpr int JJ = decltype(jj_c)::value, J = (I & 1) ? T::NI - 1 - JJ : JJ;
                            if constexpr (ACC_FILE) {
                                mma16_acc<INT8>(acc[I][J], frag_value(bc[0][J]), frag_value(ar[S][0]));
                                slot(std::integral_constant<int, FIRST + 2 * JJ>{});
                                mma16_acc<INT8>(acc[I][J], frag_value(bc[1][J]), frag_value(ar[S][1]));
                                slot(std::integral_constant<int, FIRST + 2 * JJ + 1>{});
                                if constexpr (FINAL && I > 0) {
                                    // the block of the row before that was computed at this place in its row: 2 NI
                                    // matrix instructions ago, its result has long been written
                                    constexpr int JP = ((I - 1) & 1) ? T::NI - 1 - JJ : JJ;
                                    // (the loads that the step before issued, all beyond the end of K, are the last
                                    // to write LDS: nothing but stores is in flight when the wave ends)
                                    if constexpr (I == 1 && JJ == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                                    store_from_acc<64 * JP>(early, acc[I - 1][JP]);
                                    if constexpr (JJ == T::NI - 1) early += early_step;
                                }
                            } else {
                                acc[I][J] = Acc<INT8, 16>::mma(frag_value(bc[0][J]), frag_value(ar[S][0]), acc[I][J]);
                                acc[I][J] = Acc<INT8, 16>::mma(frag_value(bc[1][J]), frag_value(ar[S][1]), acc[I][J]);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        });
                    };
                    constexpr int HALF = 4 + NRB + (L_HI - L_LO + 1) / 2;
                    if constexpr (REAL0) row(std::integral_constant<int, R0>{}, Zero{});
                    if constexpr (!ACC_FILE) {
                        static_for<HALF>([&](auto k_c) { item(k_c); });
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    row(std::integral_constant<int, R1>{}, std::integral_constant<int, REAL0 ? PER_ROW : 0>{});
                    if constexpr (!ACC_FILE) {
                        static_for<NITEMS - HALF>([&](auto k_c) { item(std::integral_constant<int, HALF + decltype(k_c)::value>{}); });
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr (G == LAST - 1 && !FINAL) {
                        // K step kt+1 has landed; this step's A loads (for step kt+2) may stay in flight
#ifdef XP_TRACE
                        const long long tb0 = clock64();
                        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(T::IA));
                        const long long tb1 = clock64();
                        __builtin_amdgcn_s_barrier();
                        tr_wait[0] += tb1 - tb0;
                        tr_wait[1] += clock64() - tb1;
#else
                        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(T::IA));
                        __builtin_amdgcn_s_barrier();
#endif
                    }
                });
                if constexpr (POS < 0) {
                    const int a = cur_a, b = nxt_b;
                    cur_a = nxt_a; nxt_a = fill_a; fill_a = a;
                    nxt_b = fill_b; fill_b = b;
                }
            };
#ifdef XP_TRACE
            tr_c[1] = clock64(); tr_w[1] = wall_clock64();
#endif
            // steps whose loads (K step kt + 2) are whole steps inside K, in rounds after which both rings and the
            // B fragment sets are where they were: every LDS offset an instruction constant
            const int whole = p.Kb / RB - 2;
            int kt = 0;
            for (; kt + 6 <= whole; kt += 6)
                static_for<6>([&](auto pos_c) {
                    step(kt + decltype(pos_c)::value, std::integral_constant<bool, (decltype(pos_c)::value & 1) != 0>{}, std::false_type{}, pos_c,
                         std::false_type{});
                });
            bool stored = false;
            auto tail_step = [&](int k, auto odd_c) {
                if constexpr (EARLY) {
                    if (k == KT - 1 && early != nullptr) {
                        step(k, odd_c, std::true_type{}, RunTime{}, std::true_type{});
                        stored = true;
                        return;
                    }
                }
                step(k, odd_c, std::true_type{}, RunTime{}, std::false_type{});
            };
            while (kt < KT) {
                tail_step(kt, std::false_type{});
                if (++kt < KT) tail_step(kt, std::true_type{});
                ++kt;
            }
            // (the compiler does not know that the statements above are matrix instructions and leaves no room
            // between the last of them and the first read of its result)
            if constexpr (ACC_FILE) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
            if constexpr (EARLY) {
                if (stored) {
                    static_for<T::NI>([&](auto j_c) { store_from_acc<64 * decltype(j_c)::value>(early, acc[T::MI - 1][decltype(j_c)::value]); });
#ifdef XP_TRACE
                    tr_c[2] = clock64(); tr_w[2] = wall_clock64();
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
                    tr_c[3] = clock64(); tr_w[3] = wall_clock64();
                    if (p.trace && tid == 0) {
#pragma unroll
                        for (int x = 0; x < 4; ++x) { p.trace[tr_slot * 16 + x] = tr_c[x]; p.trace[tr_slot * 16 + 4 + x] = tr_w[x]; }
                        for (int x = 0; x < 3; ++x) p.trace[tr_slot * 16 + 8 + x] = tr_wait[x];
                    }
#endif
                    return;
                }
            }
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));     // no load may outlive the wave
        }
    } else
    if (KT > 0) {
        AFrag xa[T::MI], ya[T::MI];                           // fragment sets of even / odd sub-steps
        BFrag xb[T::NI], yb[T::NI];
        constexpr bool WV = ASMR;
        if constexpr (WV) {
            // woven: step j issues B(j+NS) and A(j+NSA), the deeper ring's last, and so do the steps before the first:
            // every buffer of both rings is filled before the loop
            constexpr int DEEP = T::NS > T::NSA ? T::NS : T::NSA;
#pragma unroll
            for (int j = -DEEP; j < 0; ++j) {
                if (!T::B_DEEP && j + T::NS >= 0) issue_b(j + T::NS, T::B_BASE + (j + T::NS) * T::B_BYTES, 0, T::IB, std::true_type{});
                if (j + T::NSA >= 0) issue_a(j + T::NSA, (j + T::NSA) * T::A_BYTES, 0, T::IA, std::true_type{});
                if (T::B_DEEP && j + T::NS >= 0) issue_b(j + T::NS, T::B_BASE + (j + T::NS) * T::B_BYTES, 0, T::IB, std::true_type{});
            }
        } else if constexpr (T::ASYM) {
            // step j issues B(j+NS-1) and A(j+NSA-1), the deeper ring's last; the steps before the first one do the same
            constexpr int DEEP = T::B_DEEP ? T::NS : T::NSA;
#pragma unroll
            for (int j = -(DEEP - 1); j < 0; ++j) {
                if (!T::B_DEEP && j + T::NS - 1 >= 0) issue_b(j + T::NS - 1, T::B_BASE + (j + T::NS - 1) * T::B_BYTES, 0, T::IB, std::true_type{});
                if (j + T::NSA - 1 >= 0) issue_a(j + T::NSA - 1, (j + T::NSA - 1) * T::A_BYTES, 0, T::IA, std::true_type{});
                if (T::B_DEEP) issue_b(j + T::NS - 1, T::B_BASE + (j + T::NS - 1) * T::B_BYTES, 0, T::IB, std::true_type{});
            }
        } else {
#pragma unroll
            for (int s = 0; s < T::NS - 1; ++s) issue(s, s * T::A_BYTES, T::B_BASE + s * T::B_BYTES, 0, IT, std::true_type{});
        }
        // (woven: one more K step of loads has been issued than the barrier inside a step finds)
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(WV ? PENDING + IT : PENDING));
        __builtin_amdgcn_s_barrier();
        // fragment sets alternate between sub-steps; `odd` says which set holds the sub-step that
        // is multiplied next (only for PH == 1 does it change from K step to K step)
        typedef std::integral_constant<int, -1> RunTime;
        typedef std::integral_constant<int, 0> Zero;
        typedef std::integral_constant<int, 1> One;
        if constexpr (ASMR) {
            static_for<T::MI + T::NI>([&](auto f_c) { read_frag_asm(Zero{}, std::integral_constant<int, T::B_BASE>{}, Zero{}, f_c, 0, 0, xa, xb); });
        } else {
            read_frags(0, T::B_BASE, 0, xa, xb);
        }
        int cur_a = 0, cur_b = T::B_BASE;
        int fill_a = (T::NSA - 1) * T::A_BYTES, fill_b = T::B_BASE + (T::NS - 1) * T::B_BYTES;
        // POS >= 0: the step's position in the rings as a constant (the step runs POS steps after one that
        // found both rings at their first buffers): every LDS offset becomes an instruction constant and the
        // run-time ring state is neither read nor advanced.  POS < 0: the state variables above.
        auto step = [&](int kt, auto odd_in, auto check_c, auto pos_c) {
            constexpr bool ODD = decltype(odd_in)::value;   // set multiplied in sub-step 0: false = X, true = Y
            constexpr int POS = decltype(pos_c)::value;
            constexpr int CA = POS < 0 ? -1 : (POS % T::NSA) * T::A_BYTES, NA = POS < 0 ? -1 : ((POS + 1) % T::NSA) * T::A_BYTES;
            constexpr int CB = POS < 0 ? -1 : T::B_BASE + (POS % T::NS) * T::B_BYTES;
            constexpr int NB = POS < 0 ? -1 : T::B_BASE + ((POS + 1) % T::NS) * T::B_BYTES;
            const int nxt_a = POS >= 0 ? NA : (cur_a + T::A_BYTES == A_END ? 0 : cur_a + T::A_BYTES);
            const int nxt_b = POS >= 0 ? NB : (cur_b + T::B_BYTES == B_END ? T::B_BASE : cur_b + T::B_BYTES);
            const int now_a = POS >= 0 ? CA : cur_a, now_b = POS >= 0 ? CB : cur_b;
            // loads go into the buffers read in step kt-1
            const int into_a = POS >= 0 ? ((POS + T::NSA - 1) % T::NSA) * T::A_BYTES : fill_a;
            const int into_b = POS >= 0 ? T::B_BASE + ((POS + T::NS - 1) % T::NS) * T::B_BYTES : fill_b;
            if constexpr (ASMR) {
                // (issued in the second sub-step, below)
            } else if constexpr (T::ASYM) {
                if constexpr (!T::B_DEEP) issue_b(kt + T::NS - 1, into_b, 0, T::IB, check_c);
                issue_a(kt + T::NSA - 1, into_a, 0, T::IA, check_c);
                if constexpr (T::B_DEEP) issue_b(kt + T::NS - 1, into_b, 0, T::IB, check_c);
            } else if constexpr (!T::SPREAD) {
                issue(kt + T::NS - 1, into_a, into_b, 0, IT, check_c);
            }
            if constexpr (ASMR) {
                // two sub-steps: the second one's fragments (set Y) are read while the first is multiplied
                static_assert(T::PH == 2 && !ODD && !T::SPREAD, "assembly reads: two sub-steps per K step");
                // The barrier in the middle of the step is passed when every wave has read the current buffers
                // for the last time, so the second sub-step refills them: with the loads for K step kt + NS
                // (A: kt + NSA), a share behind each block row.  They have a whole K step to land, not half.
                weave(std::integral_constant<int, CA>{}, std::integral_constant<int, CB>{}, One{}, now_a, now_b, xa, xb, ya, yb, [](auto) {});
#ifdef XP_TRACE
                {
                    const long long tb0 = clock64();
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(PENDING));
                    const long long tb1 = clock64();
                    __builtin_amdgcn_s_barrier();
                    tr_wait[0] += tb1 - tb0;
                    tr_wait[1] += clock64() - tb1;
                }
#else
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(PENDING));
                __builtin_amdgcn_s_barrier();
#endif
                weave(std::integral_constant<int, NA>{}, std::integral_constant<int, NB>{}, Zero{}, nxt_a, nxt_b, ya, yb, xa, xb, [&](auto i_c) {
                    constexpr int I = decltype(i_c)::value;
                    constexpr int LO = I * IT / T::MI, HI = (I + 1) * IT / T::MI;
                    if constexpr (T::ASYM && !T::B_DEEP) {       // B first: the deeper ring's loads are the ones that may stay in flight
                        issue_b(kt + T::NS, now_b, LO, HI < T::IB ? HI : T::IB, check_c);
                        issue_a(kt + T::NSA, now_a, LO > T::IB ? LO - T::IB : 0, HI - T::IB, check_c);
                    } else {
                        issue_a(kt + T::NSA, now_a, LO, HI < T::IA ? HI : T::IA, check_c);
                        issue_b(kt + T::NS, now_b, LO > T::IA ? LO - T::IA : 0, HI - T::IA, check_c);
                    }
                });
            } else {
#pragma unroll
                for (int ph = 0; ph < T::PH - 1; ++ph) {
                    if constexpr (T::SPREAD) issue(kt + T::NS - 1, into_a, into_b, ph * IT / T::PH, (ph + 1) * IT / T::PH, check_c);
                    const bool cur_is_y = ((ph & 1) != 0) != ODD;
                    if (cur_is_y) read_frags(now_a, now_b, ph + 1, xa, xb);
                    else read_frags(now_a, now_b, ph + 1, ya, yb);
                    __builtin_amdgcn_sched_barrier(0);
                    if (cur_is_y) mma_all(ya, yb);
                    else mma_all(xa, xb);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // last sub-step: its fragments were read before the barrier, the MFMAs run after it
                constexpr bool LAST_IS_Y = (((T::PH - 1) & 1) != 0) != ODD;
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(T::SPREAD ? PENDING - (IT - (T::PH - 1) * IT / T::PH) : PENDING));
                __builtin_amdgcn_s_barrier();
                if constexpr (T::SPREAD) issue(kt + T::NS - 1, into_a, into_b, (T::PH - 1) * IT / T::PH, IT, check_c);
                // sub-step 0 of the next buffers (zeros after the last step, never multiplied)
                if constexpr (LAST_IS_Y) read_frags(nxt_a, nxt_b, 0, xa, xb);
                else read_frags(nxt_a, nxt_b, 0, ya, yb);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (LAST_IS_Y) mma_all(ya, yb);
                else mma_all(xa, xb);
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (POS < 0) {
                fill_a = cur_a;
                fill_b = cur_b;
                cur_a = nxt_a;
                cur_b = nxt_b;
            }
        };
#ifdef XP_TRACE
        tr_c[1] = clock64(); tr_w[1] = wall_clock64();
#endif
        if constexpr (T::PH % 2 == 0) {
            // steps whose loads (for step kt + NS - 1, A possibly one further) are whole steps inside K
            constexpr int AHEAD = (T::NSA > T::NS ? T::NSA : T::NS) - (WV ? 0 : 1);
            const int whole = p.Kb / RB - AHEAD;
            int kt = 0;
            if constexpr (ASMR) {
                // the main part of the loop in rounds of ROUND steps, after which both rings are where they were
                constexpr int ROUND = T::NSA == T::NS ? T::NS : T::NSA * T::NS;
                for (; kt + ROUND <= whole; kt += ROUND)
                    static_for<ROUND>([&](auto pos_c) { step(kt + decltype(pos_c)::value, std::false_type{}, std::false_type{}, pos_c); });
            }
            for (; kt < whole; ++kt) step(kt, std::false_type{}, std::false_type{}, RunTime{});
            for (; kt < KT; ++kt) step(kt, std::false_type{}, std::true_type{}, RunTime{});
        } else {
            // an odd number of sub-steps per K step: the roles of the two sets swap every step
            int kt = 0;
            for (; kt + 1 < KT; kt += 2) {
                step(kt, std::false_type{}, std::true_type{}, RunTime{});
                step(kt + 1, std::true_type{}, std::true_type{}, RunTime{});
            }
            if (kt < KT) step(kt, std::false_type{}, std::true_type{}, RunTime{});
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));     // no load may outlive the wave
    }
#ifdef XP_TRACE
    tr_c[2] = clock64(); tr_w[2] = wall_clock64();
#endif

    // epilogue
    using OutT = typename std::conditional<INT8, int, float>::type;
    OutT *C = (OutT *)p.C + batch * p.strideC;
    if constexpr (MF == 16 && !PLANAR) {
        // A tile that lies inside the matrix, beta == 0, 16-byte aligned rows: one address per lane for the whole wave
        // tile (the block row adds a multiple of the pitch, the block column is an instruction constant), no test per
        // block, and with alpha == 1 (or integers) the accumulators are stored as they are
        const bool whole = m0 + T::BM <= m_end && n0 + T::BN <= p.N && (INT8 || p.beta == 0.0f) &&
                           (((unsigned long long)C | (unsigned long long)(p.ldc * (long long)sizeof(OutT))) & 15) == 0;
        if (whole) {
            typedef OutT out4 __attribute__((ext_vector_type(4)));
            OutT *base = C + (long long)(m0 + wm * T::WTM + (lane & 15)) * p.ldc + (n0 + wn * T::WTN + (lane >> 4) * 4);
            const long long step16 = 16 * p.ldc;
            // (the stores below are assembly text to the compiler: it does not see that they read what the last matrix
            // instructions write, and a tile of one or two blocks per wave has nothing else in between)
            if constexpr (!T::NTSTORE) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
            if (INT8 || p.alpha == 1.0f) {
                if constexpr (T::PAIR != 0 && T::NWAVE == 4 && !T::NTSTORE) {
                    // accumulators that live in the accumulation registers go to memory from there (the compiler would
                    // first copy all 256 of them to vector registers: a thousand cycles before the first store)
                    static_for<T::MI * T::NI>([&](auto b_c) {
                        constexpr int I = decltype(b_c)::value / T::NI, J = decltype(b_c)::value % T::NI;
                        store_from_acc<64 * J>(base, acc[I][J]);
                        if constexpr (J == T::NI - 1) base += step16;
                    });
                } else {
#pragma unroll
                    for (int i = 0; i < T::MI; ++i, base += step16)
#pragma unroll
                        for (int j = 0; j < T::NI; ++j)
                            put_tile<T::NTSTORE>((out4 *)(base + 16 * j), out4{(OutT)acc[i][j][0], (OutT)acc[i][j][1], (OutT)acc[i][j][2], (OutT)acc[i][j][3]});
                }
            } else {
                if constexpr (!INT8) {
#pragma unroll
                    for (int i = 0; i < T::MI; ++i, base += step16)
#pragma unroll
                        for (int j = 0; j < T::NI; ++j)
                            put_tile<T::NTSTORE>((out4 *)(base + 16 * j),
                                                 out4{p.alpha * acc[i][j][0], p.alpha * acc[i][j][1], p.alpha * acc[i][j][2], p.alpha * acc[i][j][3]});
                }
            }
#ifdef XP_TRACE
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            tr_c[3] = clock64(); tr_w[3] = wall_clock64();
            if (p.trace && tid == 0) {
#pragma unroll
                for (int x = 0; x < 4; ++x) { p.trace[tr_slot * 16 + x] = tr_c[x]; p.trace[tr_slot * 16 + 4 + x] = tr_w[x]; }
                for (int x = 0; x < 3; ++x) p.trace[tr_slot * 16 + 8 + x] = tr_wait[x];
            }
#endif
            return;
        }
    }
#pragma unroll
    for (int i = 0; i < T::MI; ++i)
#pragma unroll
        for (int j = 0; j < T::NI; ++j) {
            if constexpr (MF == 32)
                store_block32<INT8, T::NTSTORE>(acc[i][j], C, p.ldc, m0 + wm * T::WTM + i * 32, n0 + wn * T::WTN + j * 32, lane, m_end,
                                    p.N, p.alpha, p.beta);
            else if constexpr (PLANAR)
                store_block16t_planar(acc[i][j], C, p.c_plane, m0 + wm * T::WTM + i * 16, n0 + wn * T::WTN + j * 16, lane, m_end,
                                      p.N, p.alpha);
            else
                store_block16t<INT8, T::NTSTORE>(acc[i][j], C, p.ldc, m0 + wm * T::WTM + i * 16, n0 + wn * T::WTN + j * 16, lane, m_end,
                                     p.N, p.alpha, p.beta);
        }
#ifdef XP_TRACE
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));         // the stores have reached L2
    tr_c[3] = clock64(); tr_w[3] = wall_clock64();
    if (p.trace && tid == 0) {
#pragma unroll
        for (int x = 0; x < 4; ++x) { p.trace[tr_slot * 16 + x] = tr_c[x]; p.trace[tr_slot * 16 + 4 + x] = tr_w[x]; }
        for (int x = 0; x < 3; ++x) p.trace[tr_slot * 16 + 8 + x] = tr_wait[x];
    }
#endif
}

template <bool INT8, class T, int MODE>
__global__ __launch_bounds__(T::NT, T::OCC) void dl_kernel(DlParams p)
{
    __shared__ __attribute__((aligned(1024))) char lds[T::LDS];
    dl_body<INT8, T, MODE>(p, lds, blockIdx.x, 0, p.M, p.tiles_m);
}

// Two tile heights in one launch: full rounds of T1 tiles first, then one last round of the lower
// T2 tiles, so that a grid that does not fill its last round of compute units wastes less of it
// (workgroups start in index order: the T1 tiles occupy every compute unit before a T2 tile starts).
template <bool INT8, class T1, class T2, int MODE>
__global__ __launch_bounds__(T1::NT, 1) void dl_kernel_two_heights(DlParams p)
{
    static_assert(T1::NT == T2::NT && T1::BN == T2::BN, "the two tile types share the workgroup shape and the tile width");
    __shared__ __attribute__((aligned(1024))) char lds[T1::LDS > T2::LDS ? T1::LDS : T2::LDS];
    if ((int)blockIdx.x < p.n1) dl_body<INT8, T1, MODE>(p, lds, blockIdx.x, 0, p.m_split, p.tiles_m);
    else dl_body<INT8, T2, MODE>(p, lds, blockIdx.x - p.n1, p.m_split, p.M, p.tiles_m2);
}

// The same two tile heights when one round of each covers the problem (at most one workgroup per compute unit):
// workgroup i computes T1 tile i and then, without leaving the compute unit, T2 tile i.  Against two workgroups
// one after the other this saves the hand-over (3.5 us between the last store of the first and the entry of the
// second, measured with time stamps in the kernel), and the second tile's set-up and first loads run while the
// first tile's stores drain.
template <bool INT8, class T1, class T2, int MODE>
__global__ __launch_bounds__(T1::NT, 1) void dl_kernel_pair(DlParams p)
{
    static_assert(T1::NT == T2::NT && T1::BN == T2::BN, "the two tile types share the workgroup shape and the tile width");
    __shared__ __attribute__((aligned(1024))) char lds[T1::LDS > T2::LDS ? T1::LDS : T2::LDS];
    dl_body<INT8, T1, MODE>(p, lds, blockIdx.x, 0, p.m_split, p.tiles_m);
    if ((int)blockIdx.x < p.tiles_m2 * p.tiles_n) {
        __builtin_amdgcn_s_barrier();                    // every wave has left the first tile's K loop: its LDS buffers may be refilled
        dl_body<INT8, T2, MODE>(p, lds, blockIdx.x, p.m_split, p.M, p.tiles_m2);
    }
}

// ------------------------------------------------------------------------------------ host side

template <bool INT8>
bool dl_can_run_common(const Problem &q, int BM, int BN, int RB, int MF)
{
    // planar output: the 16x16 blocks' lanes hold 16 consecutive rows of a column, a contiguous run of a plane
    if (q.c_plane && (MF != 16 || q.beta != 0.0f || INT8)) return false;
    const int64_t esz = INT8 ? 1 : 2;
    if (q.in_type != (INT8 ? XP_I8 : XP_BF16)) return false;
    if (q.K <= 0) return false;
    if ((q.K * esz) % 16 != 0) return false;
    if (q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.K * esz > 0x3fffffffLL) return false;
    if (q.batch > 65535) return false;
    if (q.b_sk != 1 || (q.b_sn * esz) % 16 != 0 || ((uintptr_t)q.B % 16) != 0) return false;
    if ((q.strideB * esz) % 16 != 0) return false;
    if ((BN - 1) * q.b_sn * esz + q.K * esz >= 0x7fffffffLL) return false;
    if (q.conv) {
        if (INT8) return false;
        const int64_t in_bytes = (q.M / (q.P * q.Q)) * q.H * q.W * q.Cin * esz;
        // offsets are taken from (-pad_h, -pad_w) of the first image; a lane's taps are one bit each of a 32-bit mask
        if (in_bytes + (q.ph * q.W + q.pw) * q.Cin * esz >= 0x7fffffffLL) return false;
        if (q.R * q.S > 32) return false;
        if ((q.Cin * esz) % RB != 0) return false;         // a K step never straddles a filter tap
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
DlParams dl_params(const Problem &q)
{
    const int64_t esz = INT8 ? 1 : 2;
    DlParams p;
    p.A = (const char *)q.A; p.B = (const char *)q.B; p.C = (char *)q.C;
    p.M = (int)q.M; p.N = (int)q.N;
    p.Kb = (int)(q.K * esz);
    p.KT = (p.Kb + T::RB - 1) / T::RB;
    p.lda_b = q.a_sm * esz; p.ldb_b = q.b_sn * esz;
    p.ldc = q.ldc;
    p.c_plane = q.c_plane;
    p.strideA_b = q.strideA * esz; p.strideB_b = q.strideB * esz; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    p.tiles_m = (int)((q.M + T::BM - 1) / T::BM);
    p.tiles_n = (int)((q.N + T::BN - 1) / T::BN);
    // tile-rows per raster group; XP_GROUP_M overrides it for tuning experiments
    static const int env_group_m = [] { const char *e = getenv("XP_GROUP_M"); return e ? atoi(e) : 0; }();
    p.group_m = env_group_m > 0 ? env_group_m : 4;
    p.in_bytes = 0; p.H = p.W = p.Cin_b = p.R = p.S = p.PQ = p.Q = p.sh = p.sw = p.ph = p.pw = 0;
    p.pq_magic = p.q_magic = 0; p.pq_shift = p.q_shift = 0; p.tap_rep = 0;
    if (q.conv) {
        p.in_bytes = (unsigned)((q.M / (q.P * q.Q)) * q.H * q.W * q.Cin * esz);
        p.H = (int)q.H; p.W = (int)q.W; p.Cin_b = (int)(q.Cin * esz); p.R = (int)q.R; p.S = (int)q.S;
        p.PQ = (int)(q.P * q.Q); p.Q = (int)q.Q;
        auto magic = [](int d, unsigned &m, int &sh) {
            sh = 0;
            while ((1LL << sh) < d) ++sh;
            m = (unsigned)((((unsigned long long)1 << (31 + sh)) + (unsigned)d - 1) / (unsigned)d);
        };
        magic(p.PQ, p.pq_magic, p.pq_shift);
        magic(p.Q, p.q_magic, p.q_shift);
        for (int r = 0; r < p.R; ++r) p.tap_rep |= 1u << (r * p.S);
        p.sh = (int)q.sh; p.sw = (int)q.sw; p.ph = (int)q.ph; p.pw = (int)q.pw;
    }
    p.n1 = 0; p.m_split = 0; p.tiles_m2 = 0;
#ifdef XP_TRACE
    p.trace = g_dl_trace;
#endif
    return p;
}

template <bool INT8, class T>
hipError_t dl_launch(const Problem &q)
{
    const DlParams p = dl_params<INT8, T>(q);
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)q.batch);
    if constexpr (T::MF == 16 && !INT8) {
        if (q.conv && q.c_plane) {
            hipLaunchKernelGGL((dl_kernel<INT8, T, 2>), grid, dim3(T::NT), 0, q.stream, p);
            return hipGetLastError();
        }
    }
    if (q.conv) hipLaunchKernelGGL((dl_kernel<INT8, T, 1>), grid, dim3(T::NT), 0, q.stream, p);
    else hipLaunchKernelGGL((dl_kernel<INT8, T, 0>), grid, dim3(T::NT), 0, q.stream, p);
    return hipGetLastError();
}

// Rows [0, m_split) in whole rounds of T1 tiles over the 256 compute units, the rest in T2 tiles:
// as few T1 rounds as leave a remainder that one round of T2 tiles covers.
template <class T1, class T2>
int64_t two_heights_split(const Problem &q)
{
    const int64_t tiles_n = (q.N + T1::BN - 1) / T1::BN;
    const int64_t per_round = tiles_n >= 256 ? 1 : 256 / tiles_n;          // tile-rows that one round holds
    const int64_t rows1 = per_round * T1::BM, cap2 = per_round * T2::BM;
    if (q.M <= cap2) return 0;
    const int64_t k = (q.M - cap2 + rows1 - 1) / rows1;
    return k * rows1 < q.M ? k * rows1 : q.M;
}

template <bool INT8, class T1, class T2, bool ASM = false>
hipError_t dl_launch_two_heights(const Problem &q)
{
    constexpr int M0 = ASM ? 6 : 0;                        // the modes with assembly reads follow the plain ones
    DlParams p = dl_params<INT8, T1>(q);
    const int64_t split = two_heights_split<T1, T2>(q);
    p.m_split = (int)split;
    p.tiles_m = (int)(split / T1::BM);                    // split is a multiple of T1::BM or equals M
    if (split % T1::BM != 0) p.tiles_m += 1;
    p.tiles_m2 = (int)((q.M - split + T2::BM - 1) / T2::BM);
    p.n1 = p.tiles_m * p.tiles_n;
    const int n2 = p.tiles_m2 * p.tiles_n;
    if (q.batch == 1 && p.n1 <= 256 && n2 > 0 && n2 <= p.n1) {
        // one round of each height: the two tiles of a compute unit in one workgroup
        const dim3 pgrid((unsigned)p.n1, 1);
        if constexpr (T1::MF == 16 && !INT8) {
            if (q.conv && q.c_plane) {
                hipLaunchKernelGGL((dl_kernel_pair<INT8, T1, T2, M0 + 2>), pgrid, dim3(T1::NT), 0, q.stream, p);
                return hipGetLastError();
            }
        }
        if (q.conv) hipLaunchKernelGGL((dl_kernel_pair<INT8, T1, T2, M0 + 1>), pgrid, dim3(T1::NT), 0, q.stream, p);
        else hipLaunchKernelGGL((dl_kernel_pair<INT8, T1, T2, M0>), pgrid, dim3(T1::NT), 0, q.stream, p);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)(p.n1 + n2), (unsigned)q.batch);
    if constexpr (T1::MF == 16 && !INT8) {
        if (q.conv && q.c_plane) {
            hipLaunchKernelGGL((dl_kernel_two_heights<INT8, T1, T2, M0 + 2>), grid, dim3(T1::NT), 0, q.stream, p);
            return hipGetLastError();
        }
    }
    if (q.conv) hipLaunchKernelGGL((dl_kernel_two_heights<INT8, T1, T2, M0 + 1>), grid, dim3(T1::NT), 0, q.stream, p);
    else hipLaunchKernelGGL((dl_kernel_two_heights<INT8, T1, T2, M0>), grid, dim3(T1::NT), 0, q.stream, p);
    return hipGetLastError();
}

template <class T>
double dl_cost(const Problem &q, double eff)
{
    return tile_cost_us(q, T::BM, T::BN, T::LDS, T::NT, eff, q.in_type == XP_I8 ? 1 : 2);
}


// ---- operands contiguous along their outer index (MODE 3, 4, 5 of dl_body): bf16 GEMM and batched GEMM
// with a row-major B, a column-major A, or both

inline bool dl_outer_can_run(const Problem &q, int BM, int BN, bool amm, bool bnm)
{
    if (q.in_type != XP_BF16 || q.conv || q.c_plane) return false;
    if (q.K <= 0 || q.M > 0x7fffffffLL || q.N > 0x7fffffffLL || q.batch > 65535) return false;
    if (((uintptr_t)q.A % 16) != 0 || ((uintptr_t)q.B % 16) != 0 || (q.strideA * 2) % 16 != 0 || (q.strideB * 2) % 16 != 0) return false;
    // along the outer index: whole 16-byte chunks of a k row; the K position of a step travels as a 32-bit byte offset.
    // along K: whole 16-byte chunks of a row of the operand
    if (amm) {
        if (q.a_sm != 1 || (q.a_sk * 2) % 16 != 0 || q.M % 8 != 0 || (q.K + 256) * q.a_sk * 2 >= 0x7fffffffLL) return false;
    } else {
        if (q.a_sk != 1 || (q.a_sm * 2) % 16 != 0 || q.K % 8 != 0 || (BM - 1) * q.a_sm * 2 + q.K * 2 >= 0x7fffffffLL) return false;
    }
    if (bnm) {
        if (q.b_sn != 1 || (q.b_sk * 2) % 16 != 0 || q.N % 8 != 0 || (q.K + 256) * q.b_sk * 2 >= 0x7fffffffLL) return false;
    } else {
        if (q.b_sk != 1 || (q.b_sn * 2) % 16 != 0 || q.K % 8 != 0 || (BN - 1) * q.b_sn * 2 + q.K * 2 >= 0x7fffffffLL) return false;
    }
    return q.K * 2 <= 0x3fffffffLL;
}

template <class T, int MODE>
hipError_t dl_outer_launch(const Problem &q)
{
    constexpr bool AMM = MODE == 4 || MODE == 5, BNM = MODE == 3 || MODE == 5;
    static_assert(!BNM || (T::BN * 2 <= 1024 && 1024 % (T::BN * 2) == 0 && T::BNP == T::BN), "a wave-level load fills whole k rows of the B tile");
    static_assert(!AMM || (T::BM * 2 <= 1024 && 1024 % (T::BM * 2) == 0 && T::BMP == T::BM), "a wave-level load fills whole k rows of the A tile");
    DlParams p = dl_params<false, T>(q);
    if (AMM) p.lda_b = q.a_sk * 2;                         // bytes from one k row to the next
    if (BNM) p.ldb_b = q.b_sk * 2;
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)q.batch);
    hipLaunchKernelGGL((dl_kernel<false, T, MODE>), grid, dim3(T::NT), 0, q.stream, p);
    return hipGetLastError();
}

// ---- the K-contiguous kernels with assembly reads (MODE 6, 7, 8 of dl_body)

template <bool INT8, class T>
hipError_t dl_asm_launch(const Problem &q)
{
    const DlParams p = dl_params<INT8, T>(q);
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)q.batch);
    if constexpr (!INT8) {
        if (q.conv) {
            if (q.c_plane) hipLaunchKernelGGL((dl_kernel<INT8, T, 8>), grid, dim3(T::NT), 0, q.stream, p);
            else hipLaunchKernelGGL((dl_kernel<INT8, T, 7>), grid, dim3(T::NT), 0, q.stream, p);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((dl_kernel<INT8, T, 6>), grid, dim3(T::NT), 0, q.stream, p);
    return hipGetLastError();
}

// ---- the two k sub-steps of a block back to back (DlTile::PAIR): GEMM and batched GEMM
template <bool INT8, class T>
hipError_t dl_pair_launch(const Problem &q)
{
    const DlParams p = dl_params<INT8, T>(q);
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)q.batch);
    hipLaunchKernelGGL((dl_kernel<INT8, T, 6>), grid, dim3(T::NT), 0, q.stream, p);
    return hipGetLastError();
}

// two tile heights: 224-row tiles in whole rounds, a last round of 192-row tiles
typedef DlTile<224, 256, 2, 4, 2, 128, false, 1, 16, false, 3> TwoHi;
typedef DlTile<192, 256, 2, 4, 2, 128, false, 1, 16, false, 3> TwoLo;

}  // namespace
}  // namespace xp
