// Row-streaming MFMA kernel for (batched) bf16 GEMMs that are bound by reading A: few columns (N <= 64), a
// reduction of at most 512, B stored row-major (K x N) -- the second stage of an attention block, P.V with a head
// of 64 (Table 5 of the paper: Batch GEMM).
//
// The tiled kernels read such an A as 64 rows x 128 bytes per K step: pieces of 128 bytes a kilobyte apart, each
// 256-byte unit of memory fetched as two halves at different times.  DRAM likes that less than whole rows (a copy
// of 128-byte pieces at a 1 KB stride runs at 4.4-5.0 TB/s on this chip, one of 512-byte pieces at 5.5), and all
// workgroups of the launch load, multiply and store in step, so reads and writes do not overlap.  Here
//   * B of the problem (K x 64, at most 64 KB) is brought into LDS once per workgroup, as it lies in memory, and its
//     fragments are gathered by transposing LDS reads;
//   * every wave streams block rows of A (16 rows) of its own: a slab is 16 rows x 512 bytes (half of the longest K),
//     loaded straight into LDS by 8 loads of 1 KB that each fetch two half-rows of 512 contiguous bytes, into a ring
//     of three slabs per wave, two slabs ahead of the one being multiplied.  A wave waits only for its own loads
//     (no workgroup barrier after the start), so the waves of a compute unit drift apart and loads, MFMAs and stores
//     of different waves overlap;
//   * a block row's 16 x 64 result is stored as soon as its last slab has been multiplied.
// LDS: 64 KB (B) + 4 waves x 3 slabs x 8 KB = 160 KB, one workgroup of 256 threads per compute unit.
#include "xp_internal.hpp"
#include "xp_epilogue.hpp"
#include "xp_lds_tr.hpp"

namespace xp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr unsigned OOB = 0x80000000u;     // byte offset outside every buffer range used here
constexpr int KMAX = 512, NMAX = 64;      // extents the LDS layout holds
constexpr int BROW = NMAX * 2;            // bytes of one k row of B in LDS
constexpr int B_BYTES = KMAX * BROW;      // 64 KB
constexpr int SLAB_K = 256;               // k per slab
constexpr int SLAB_ROWB = SLAB_K * 2;     // bytes of one slab row
constexpr int SLAB_BYTES = 16 * SLAB_ROWB;
constexpr int NSLAB = 3;
constexpr int NW = 4;                     // waves per workgroup
constexpr int LDS_BYTES = B_BYTES + NW * NSLAB * SLAB_BYTES;
static_assert(LDS_BYTES == 160 * 1024, "the layout fills the LDS of a compute unit exactly");

struct RsParams {
    const char *A, *B;
    float *C;
    int M, N, Kb;                          // Kb: K in bytes
    int rows_per_wg;                       // multiple of 64
    long long lda_b, ldb_b, ldc;
    long long strideA_b, strideB_b, strideC;
    float alpha, beta;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// chunk swizzle of a 128-byte k row of B for the transposing reads (the same term as the tiled kernels use for
// rows of 128 bytes): a read touches the 16 rows 8g + q (+4), g, q = 0..3, 32 bytes each
__device__ __forceinline__ int b_swz(int kr) { return (((kr >> 1) & 1) | (((kr >> 3) & 1) << 1)) << 1; }

__global__ __launch_bounds__(NW * 64, 1) void rs_kernel(RsParams p)
{
    __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // all workgroups of a problem on one XCD: its B is fetched into one L2
    unsigned bx, by;
    xcd_batch_remap(bx, by);
    const long long batch = by;
    const int r0 = (int)bx * p.rows_per_wg;                             // first row of this workgroup
    const int m_end = min(p.M, r0 + p.rows_per_wg);
    const int rows = m_end - r0;
    if (rows <= 0) return;                                              // (uniform: the whole workgroup)
    const int Kb = __builtin_amdgcn_readfirstlane(p.Kb);
    const int halves = Kb > SLAB_ROWB ? 2 : 1;
    const int lda_b = __builtin_amdgcn_readfirstlane((int)p.lda_b);

    const __amdgpu_buffer_rsrc_t ra = make_rsrc(p.A + batch * p.strideA_b + (long long)r0 * p.lda_b,
                                                (unsigned)((long long)(rows - 1) * p.lda_b + Kb));
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(p.B + batch * p.strideB_b, (unsigned)((long long)(Kb / 2 - 1) * p.ldb_b + p.N * 2));

    // ---- B into LDS: a wave-level load fills 8 k rows of 128 bytes; the lane at chunk position pc of k row kr
    // fetches chunk pc ^ swizzle(kr) (a chunk: 8 columns); rows past K and chunks past N are out of range (zeros)
#pragma unroll
    for (int i = 0; i < KMAX / 8 / NW; ++i) {
        const int kr = (wave + i * NW) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ b_swz(kr);
        const unsigned off = ((kr * 2 < Kb) & (chunk * 8 < p.N)) ? (unsigned)(kr * p.ldb_b) + (chunk << 4) : OOB;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void *)(lds + (wave + i * NW) * 1024), 16, off, 0, 0, 0);
    }

    // ---- A slabs.  Load i of a slab fills slab rows 2i and 2i + 1: lane l lands at row 2i + (l >> 5), position
    // l & 31, and fetches the chunk whose swizzled position that is (chunk ^ row: the 16 rows x 4 k groups of a
    // fragment read then fall into 16 different bank groups in every pass of the read)
    char *const slabs = lds + B_BYTES + wave * (NSLAB * SLAB_BYTES);
    unsigned a_off[8];                                                  // byte offset of the lane's chunk: row and position within the half row
    int a_chunk[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = 2 * i + (lane >> 5);
        a_chunk[i] = (lane & 31) ^ row;
        a_off[i] = (unsigned)(row * lda_b) + (a_chunk[i] << 4);
    }
    const int my_block_rows = (rows + 16 * NW - 1 - 16 * wave) / (16 * NW);   // block rows wave, wave + NW, ... below `rows`
    const int ntask = my_block_rows * halves;
    // task t: half t % halves of this wave's block row t / halves.  Always 8 loads: past the end they are out of
    // range (zeros, no memory touched), which keeps the count of loads in flight the same in every step.
    auto issue_task = [&](int t, int slab) {
        const int br = t / halves, h = t - br * halves;
        const int row0 = (wave + br * NW) * 16;                         // within the workgroup's rows
        const unsigned base = (unsigned)(row0 * lda_b) + h * SLAB_ROWB;
        const bool live = t < ntask;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // rows past the workgroup's last row and chunks past K are sent out of range explicitly (the scalar
            // part of the address takes no part in the buffer's range check)
            const bool ok = live & (row0 + 2 * i + (lane >> 5) < rows) & (h * SLAB_ROWB + (a_chunk[i] << 4) < Kb);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void *)(slabs + slab * SLAB_BYTES + i * 1024), 16, ok ? a_off[i] : OOB,
                                                     (int)base, 0, 0);
        }
    };
    issue_task(0, 0);
    issue_task(1, 1);
    // this wave's part of B has landed (the 16 slab loads behind it may be in flight); then everybody's
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    __syncthreads();

    // fragment read addresses.  A: lane l reads row l & 15, k group l >> 4 of k step j: chunk 4j + (l >> 4), swizzled.
    const unsigned lds_base = lds_address(lds);
    unsigned fa[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) fa[j] = lds_address(slabs) + (lane & 15) * SLAB_ROWB + (((4 * j + (lane >> 4)) ^ (lane & 15)) << 4);
    // B (transposing reads): lane a = l%16 of block g = l/16 addresses k row 8g + (a >> 2) (+ 32 per k step, + 4 for the
    // second read), the 8 bytes at columns 16 jn + 4 (a & 3)
    unsigned fb[4];
    {
        const int a16 = lane & 15, kr = 8 * (lane >> 4) + (a16 >> 2);
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) {
            const int chunk = 2 * jn + ((a16 & 3) >> 1);
            fb[jn] = lds_base + kr * BROW + ((chunk ^ b_swz(kr)) << 4) + 8 * (a16 & 1);
        }
    }

    f32x4 acc[4];
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) acc[jn] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    float *const C = p.C + batch * p.strideC;

    int slab = 0;
    for (int t = 0; t < ntask; ++t) {
        const int br = t / halves, h = t - br * halves;
        int into = slab + 2;
        if (into >= NSLAB) into -= NSLAB;
        issue_task(t + 2, into);                                        // into the slab multiplied in the step before
        // this task's 8 loads have landed; the 16 of the two tasks behind it (and nothing else) may be in flight
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        const unsigned a_at = slab * SLAB_BYTES;
        const unsigned b_at = h * (SLAB_K * BROW);
        u32x4 af[2];
        FragHalves bf[2][4];
        auto read_step = [&](auto j_c, int set) {
            constexpr int J = decltype(j_c)::value;
            af[set] = lds_read_b128<0>(fa[J] + a_at);
#pragma unroll
            for (int jn = 0; jn < 4; ++jn) {
                bf[set][jn].lo = lds_read_tr16_b64<J * 32 * BROW>(fb[jn] + b_at);
                bf[set][jn].hi = lds_read_tr16_b64<J * 32 * BROW + 4 * BROW>(fb[jn] + b_at);
            }
        };
        read_step(std::integral_constant<int, 0>{}, 0);
        static_for<8>([&](auto j_c) {
            constexpr int J = decltype(j_c)::value;
            constexpr int S = J & 1;
            lds_wait<0>();                                              // step J's fragments are in
            lds_tie(af[S]);
#pragma unroll
            for (int jn = 0; jn < 4; ++jn) frag_tie(bf[S][jn]);
            if constexpr (J + 1 < 8) read_step(std::integral_constant<int, J + 1>{}, S ^ 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int jn = 0; jn < 4; ++jn)
                acc[jn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, frag_value(bf[S][jn])),
                                                                  __builtin_bit_cast(bf16x8, af[S]), acc[jn], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
        if (h == halves - 1) {
            const int row0 = r0 + (wave + br * NW) * 16;
#pragma unroll
            for (int jn = 0; jn < 4; ++jn) {
                store_block16t<false, false>(acc[jn], C, p.ldc, row0, 16 * jn, lane, m_end, p.N, p.alpha, p.beta);
                acc[jn] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            }
        }
        slab = slab + 1 == NSLAB ? 0 : slab + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                    // no load into LDS may outlive the wave
}

// ------------------------------------------------------------------------------------ host side

bool rs_can_run(const Problem &q)
{
    if (q.in_type != XP_BF16 || q.conv || q.c_plane) return false;
    if (q.M <= 0 || q.N <= 0 || q.K <= 0 || q.N > NMAX || q.K > KMAX || q.N % 8 != 0 || q.K % 8 != 0) return false;
    if (q.a_sk != 1 || q.b_sn != 1) return false;                       // A along K, B along N
    if (((uintptr_t)q.A % 16) != 0 || ((uintptr_t)q.B % 16) != 0 || ((uintptr_t)q.C % 4) != 0) return false;
    if ((q.a_sm * 2) % 16 != 0 || (q.b_sk * 2) % 16 != 0 || (q.strideA * 2) % 16 != 0 || (q.strideB * 2) % 16 != 0) return false;
    if (q.a_sm < q.K || q.b_sk < q.N) return false;
    if (q.M > 0x7fffffffLL || q.batch > 65535) return false;
    // byte offsets inside one workgroup's rows and inside one B stay below 2^31
    if (q.M * q.a_sm * 2 >= 0x7fffffffLL || q.K * q.b_sk * 2 >= 0x7fffffffLL) return false;
    return true;
}

// rows per workgroup: enough workgroups for every compute unit where the problem allows, 64 rows at least
int rs_rows_per_wg(const Problem &q)
{
    int64_t per_problem = 256 / q.batch;                               // workgroups a problem is cut into: one round of 256 at most
    if (per_problem < 1) per_problem = 1;
    int64_t rows = (q.M + per_problem - 1) / per_problem;
    rows = (rows + 63) / 64 * 64;
    return (int)rows;
}

hipError_t rs_launch(const Problem &q)
{
    RsParams p;
    p.A = (const char *)q.A; p.B = (const char *)q.B; p.C = (float *)q.C;
    p.M = (int)q.M; p.N = (int)q.N; p.Kb = (int)(q.K * 2);
    p.rows_per_wg = rs_rows_per_wg(q);
    p.lda_b = q.a_sm * 2; p.ldb_b = q.b_sk * 2; p.ldc = q.ldc;
    p.strideA_b = q.strideA * 2; p.strideB_b = q.strideB * 2; p.strideC = q.strideC;
    p.alpha = q.alpha; p.beta = q.beta;
    const unsigned per_problem = (unsigned)((q.M + p.rows_per_wg - 1) / p.rows_per_wg);
    hipLaunchKernelGGL(rs_kernel, dim3(per_problem, (unsigned)q.batch), dim3(NW * 64), 0, q.stream, p);
    return hipGetLastError();
}

// Memory-bound estimate, on the cautious side: measured, this kernel ties with the tiled ones on the shapes it was
// written for (96 x 512 x 64 x 512: 16.6 us against 16.5) and wins only on very tall single problems, so the
// estimate leaves the choice to the table of tuned shapes and the run-time tuner.
double rs_cost(const Problem &q)
{
    if (q.M * q.batch < 64 * 128) return 1e30;
    const double bytes = (double)q.batch * ((double)q.M * q.K * 2 + (double)q.K * q.N * 2 + (double)q.M * q.N * 4);
    return 5.0 + bytes / 4.0e6;
}

const Variant kBfRowStream = {"bf16 row-streaming 16-row slabs x 512B, B resident in LDS, transposing reads, mfma16",
                              rs_can_run, rs_launch, rs_cost};

}  // namespace

int rs_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type != XP_BF16) return 0;
    out[0] = &kBfRowStream;
    return 1;
}

}  // namespace xp
