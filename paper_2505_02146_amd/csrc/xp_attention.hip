// Fused scaled dot-product attention (Table 5 of the paper: Self Attention):
//   O = softmax_over_keys(scale * Q K^T) V      for every batch index, no mask.
// The score matrix never reaches memory: a workgroup owns 64 queries, walks the keys in tiles of
// 64 and keeps, per query, a running maximum, a running sum and an unnormalised output row that
// are rescaled whenever the maximum grows (the usual streaming form of the softmax, which
// reaches the same quotient as the two-pass definition).
//
// Two kernels:
//   general   one wave per query, fp32 VALU arithmetic, any head size, fp32 or bf16 inputs
//   mfma      bf16 inputs, head size 64 for Q/K and for V: both contractions on the 16x16x32
//             matrix-core instruction, laid out so that nothing has to be transposed between them
#include "xp_internal.hpp"
#include "xp_lds_tr.hpp"

namespace xp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr unsigned OOB = 0x80000000u;
constexpr float LOG2E = 1.4426950408889634f;

struct AttnParams {
    const char *Q, *K, *V;
    float *O;
    int Lq, Lk, d, dv;
    long long ldq, ldk, ldv, ldo;                 // general kernel: elements; mfma kernel: bytes (ldo: elements)
    long long strideQ, strideK, strideV, strideO;
    float scale;
};

// ---------------------------------------------------------------------------------- general kernel

template <class T> __device__ __forceinline__ float widen(const T *p, long long i);
template <> __device__ __forceinline__ float widen<float>(const float *p, long long i) { return p[i]; }
template <> __device__ __forceinline__ float widen<unsigned short>(const unsigned short *p, long long i)
{
    return __uint_as_float((unsigned)p[i] << 16);
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// One wave per (query, batch, block of 64 output columns).  Keys are taken in chunks of CHUNK:
// the lanes share out the scores of a chunk and park them in LDS, then every lane walks the whole
// chunk for its own output column.
constexpr int CHUNK = 1024;

template <class T>
__global__ __launch_bounds__(64) void attn_general_kernel(AttnParams p)
{
    __shared__ float sc[CHUNK];
    const int lane = threadIdx.x, i = blockIdx.x;
    const long long b = blockIdx.y;
    const int x = blockIdx.z * 64 + lane;
    const T *Q = (const T *)p.Q + b * p.strideQ + (long long)i * p.ldq;
    const T *K = (const T *)p.K + b * p.strideK;
    const T *V = (const T *)p.V + b * p.strideV;

    float top = -INFINITY, total = 0.0f, acc = 0.0f;
    for (int c0 = 0; c0 < p.Lk; c0 += CHUNK) {
        const int n = min(CHUNK, p.Lk - c0);
        float mx = -INFINITY;
        for (int j = lane; j < n; j += 64) {
            const T *k = K + (long long)(c0 + j) * p.ldk;
            float dot = 0.0f;
            for (int c = 0; c < p.d; ++c) dot = fmaf(widen(Q, c), widen(k, c), dot);
            const float s = p.scale * dot;
            sc[j] = s;
            mx = fmaxf(mx, s);
        }
        const float new_top = fmaxf(top, wave_max(mx));     // finite: the chunk holds at least one key
        const float shrink = expf(top - new_top);            // 0 on the first chunk
        total *= shrink;
        acc *= shrink;
        top = new_top;
        __syncthreads();
        for (int j = 0; j < n; ++j) {
            const float w = expf(sc[j] - top);
            total += w;
            if (x < p.dv) acc = fmaf(w, widen(V, (long long)(c0 + j) * p.ldv + x), acc);
        }
        __syncthreads();
    }
    if (x < p.dv) p.O[b * p.strideO + (long long)i * p.ldo + x] = acc / total;
}

// ------------------------------------------------------------------------------------- mfma kernel
//
// Matrix-core instruction used for both contractions (16x16x32, bf16 in, fp32 out):
//   D[m][n] += sum_k A[m][k] B[k][n];  lane l supplies A[l%16][8*(l/16) .. +8] and
//   B[8*(l/16) .. +8][l%16] and holds D[4*(l/16) + v][l%16], v = 0..3.
//
// Scores are computed transposed, S^T = K Q^T (A = key rows from LDS, B = the wave's 16 queries,
// resident in registers): lane l then holds, for ITS query l%16, the keys 16*blk + 4*(l/16) + v.
// A query's softmax statistics are therefore lane-local up to two cross-lane steps (over l/16),
// and the lane's probabilities of two key blocks are exactly the 8 values the B operand of
//   O^T = V^T P^T      (A = V^T from LDS, B = P^T from registers)
// needs, if the 32 keys of one k step are numbered: slot 8*g + e  <->  key 4*g + e (e < 4),
// key 16 + 4*g + (e - 4) (e >= 4).  V lies in LDS as it lies in memory, one key per row (it goes there
// straight from global memory, like K), and the A operand -- 8 keys of ONE output column -- is
// gathered by the transposing LDS read of this architecture (ds_read_b64_tr_b16): within a block of
// 16 lanes, lane i receives as value j the element (i & 3) of the 8 bytes addressed by lane
// 4*j + (i >> 2).  With lane a of a block addressing key row k0 + (a >> 2), columns 16x + 4*(a & 3) ..,
// lane i obtains V[k0 + j][16x + i], j = 0..3: four consecutive keys of its column.  Two such reads
// (k0 = 32h + 4g and 32h + 16 + 4g) are the 8 keys of the numbering above.  O^T comes out with the
// query in l%16 again, so the running rescale factor applies without any exchange, and a lane
// ends up with 4 consecutive output columns: one 16-byte store.
constexpr int HD = 64;                                  // head size (Q/K and V)
constexpr int BQ = 64, BK = 64;                         // queries per workgroup, keys per step
constexpr int KROW = HD * 2;                            // bytes per K row in LDS (swizzled 16-byte chunks)
constexpr int K_TILE = BK * KROW;
// V tile in LDS: the layout of the K tile (128-byte rows, the 16-byte chunk index XORed with row & 6):
// a transposing read touches 16 rows x 32 bytes, and that swizzle spreads its chunks evenly over the banks
constexpr int V_TILE = K_TILE;
constexpr float TAU = 8.0f;                             // the reference maximum may lag by this much (log2 units)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));   // round to nearest even
}

__device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// s_waitcnt immediate for "vmcnt <= n and lgkmcnt == 0" (gfx9 encoding, expcnt left open)
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4); }

// D = prefetch distance in key tiles.  Tile t+D is requested at the top of step t: its K rows go
// straight into the LDS buffer that step t-1 read (a ring of D+1 buffers), its V rows into one of
// D register sets, which is interleaved into LDS D-1 steps later, at the end of step t+D-1.  Every
// wave issues exactly 4 loads per step (tiles past the end are out of range: zeros, no memory
// touched), so "at most 4*(D-1) loads outstanding" means that tile t+1 has landed.
//
// HV = head size / 64.  A head of 128 is handled as two halves of 64 that share everything but their
// tiles: the K tile of a step is two half-tiles (dimensions 0..63 and 64..127, each in the layout
// above), S^T sums four k steps instead of two; the V tile is two half-tiles of 64 output columns,
// O^T has eight column blocks instead of four.
//
// NW = waves per workgroup (4 or 8), 16 queries each.  The K and V tiles are shared by all of them, so
// eight waves halve the LDS a query needs and let twice as many waves live on a SIMD; matrix and vector
// instructions of different waves do not overlap on this hardware (a SIMD issues one or the other:
// measured, the times add), so what more waves hide is the waiting -- barriers, LDS and load latency.
// (eight waves at head size 128: two workgroups per compute unit, i.e. four waves per SIMD, need the kernel within 128 registers)
template <int D, int HV, int NW>
__global__ __launch_bounds__(64 * NW, (NW == 8 && HV == 2) ? 4 : 1) void attn_mfma_kernel(AttnParams p)
{
    constexpr int NS = D + 1;
    constexpr int KT = K_TILE * HV, VT = V_TILE * HV;   // one step's K and V tiles
    constexpr int BPW = 8 / NW;                          // 8-row blocks of a half-tile that one wave loads
    constexpr int LPS = 2 * BPW * HV;                    // loads a wave issues per step
    constexpr int BQW = 16 * NW;                         // queries per workgroup
    __shared__ __attribute__((aligned(1024))) char lds[NS * (KT + VT)];
    char *const ks = lds, *const vs = lds + NS * KT;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    unsigned bx, by;
    xcd_batch_remap(bx, by);                            // the query tiles of one problem share an L2: K, V fetched once
    const int q0 = bx * BQW;
    const long long b = by;

    const __amdgpu_buffer_rsrc_t rq = make_rsrc(p.Q + b * p.strideQ + (long long)q0 * p.ldq,
                                                (unsigned)((long long)(min(p.Lq - q0, BQW) - 1) * p.ldq + KROW * HV));
    const __amdgpu_buffer_rsrc_t rk = make_rsrc(p.K + b * p.strideK, (unsigned)((long long)(p.Lk - 1) * p.ldk + KROW * HV));
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(p.V + b * p.strideV, (unsigned)((long long)(p.Lk - 1) * p.ldv + KROW * HV));

    // the wave's queries: B operand of S^T, two k steps per 64 head dimensions
    // The parameters the key-tile loop uses, as values computed here: a parameter the compiler chose to load again
    // inside the loop would be a scalar load, which shares its counter with the LDS reads that the loop waits for in
    // part (s_waitcnt lgkmcnt(n), n > 0, assumes in-order return, which scalar loads do not promise)
    const int ldk = __builtin_amdgcn_readfirstlane((int)p.ldk), ldv = __builtin_amdgcn_readfirstlane((int)p.ldv);
    const int Lk = __builtin_amdgcn_readfirstlane(p.Lk);
    u32x4 qf[2 * HV];
#pragma unroll
    for (int s = 0; s < 2 * HV; ++s)
        qf[s] = __builtin_amdgcn_raw_buffer_load_b128(rq, (unsigned)((wave * 16 + r) * p.ldq) + (32 * s + 8 * g) * 2, 0, 0);

    // K tile: 8 wave-level loads of 8 rows each, two per wave, straight into LDS; lane l lands at
    // row l/8, position l%8 and fetches the chunk whose swizzled position that is
    const int krow = lane >> 3;
    const int kchunk = ((lane & 7) ^ (krow & 6)) << 4;   // rows of a load start at multiples of 8: the swizzle term is the lane's
    auto issue_k = [&](int j0, int koff) {
#pragma unroll
        for (int hv = 0; hv < HV; ++hv)
#pragma unroll
            for (int i = 0; i < BPW; ++i) {
                const int blk = wave * BPW + i;
                const unsigned off = (unsigned)((j0 + blk * 8 + krow) * ldk) + hv * KROW + kchunk;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lds_void *)(ks + koff + hv * K_TILE + blk * 1024), 16, off, 0, 0, 0);
            }
    };
    // V tile: the same, from V
    auto issue_v = [&](int j0, int voff) {
#pragma unroll
        for (int hv = 0; hv < HV; ++hv)
#pragma unroll
            for (int i = 0; i < BPW; ++i) {
                const int blk = wave * BPW + i;
                const unsigned off = (unsigned)((j0 + blk * 8 + krow) * ldv) + hv * KROW + kchunk;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_void *)(vs + voff + hv * V_TILE + blk * 1024), 16, off, 0, 0, 0);
            }
    };
    // transposing fragment reads: lane a = l%16 of block g addresses key row 4g + (a >> 2) (+ 32h, + 16 for
    // the second half of the numbering), the 8 bytes at columns 16x + 4*(a & 3) of its half-tile.
    // vx[x]: the lane's byte offset within a half-tile for column block x (the swizzle makes it a
    // different register per x); half-tile, k step and second half are instruction offsets
    const int va = lane & 15;
    const int vrow = 4 * g + (va >> 2);
    const int vchunk = (va & 3) >> 1, vsw = vrow & 6;
    unsigned vx[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) vx[x] = lds_address(vs) + vrow * KROW + 8 * (va & 1) + (((2 * x + vchunk) ^ vsw) << 4);
    auto read_v = [&](unsigned at, auto slot_c, auto hv_c, auto h_c) {
        constexpr int OFF = decltype(slot_c)::value * VT + decltype(hv_c)::value * V_TILE + 32 * decltype(h_c)::value * KROW;
        FragHalves f;                                    // composed into one fragment only after the wait for it
        f.lo = lds_read_tr16_b64<OFF>(at);
        f.hi = lds_read_tr16_b64<OFF + 16 * KROW>(at);
        return f;
    };

    const float c = p.scale * LOG2E;                     // scores are kept in units of log2
    float top = -INFINITY;
    f32x4 total = {0.0f, 0.0f, 0.0f, 0.0f};              // running sum of the query's probabilities (4 copies)
    const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};   // bf16 1.0 x 8
    f32x4 acc[4 * HV];
#pragma unroll
    for (int x = 0; x < 4 * HV; ++x) acc[x] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int NT = (Lk + BK - 1) / BK;
#pragma unroll
    for (int u = 0; u < D; ++u) {
        issue_k(u * BK, u * KT);
        issue_v(u * BK, u * VT);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(LPS * (D - 1)));   // tile 0 (and the queries) have landed
    wg_barrier();

    // One key tile.  CUR: the ring slot of the tile, a constant (the loop below walks the ring in whole turns), so
    // that every LDS offset is an instruction constant; MASK: the tile may reach past the last key (only the last
    // tile can).  Both used to be decided at run time in every step: about 60 of its 160 vector instructions,
    // and vector instructions are time the matrix pipe stands still.
    auto step = [&](int t, auto mask_c, auto cur_c) {
        constexpr bool MASK = decltype(mask_c)::value;
        constexpr int cur = decltype(cur_c)::value, prev = cur == 0 ? NS - 1 : cur - 1;
        const int j0 = t * BK;
        issue_k(j0 + D * BK, prev * KT);                 // slot read one barrier ago
        issue_v(j0 + D * BK, prev * VT);
        // S^T: 4 blocks of 16 keys
        f32x4 s[4];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            s[kb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            const int row = kb * 16 + r;
#pragma unroll
            for (int h = 0; h < 2 * HV; ++h) {
                const u32x4 kf = *(const u32x4 *)(ks + cur * KT + (h >> 1) * K_TILE + row * KROW + (((4 * (h & 1) + g) ^ (row & 6)) << 4));
                s[kb] = mma(kf, qf[h], s[kb]);
            }
        }
        // keys past the end count for nothing (only the last tile can hold any): the raw score is set
        // so that its scaled value is minus infinity
        if constexpr (MASK) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (j0 + kb * 16 + 4 * g + v >= Lk) s[kb][v] = c < 0.0f ? INFINITY : -INFINITY;
        }
        // largest scaled score of the tile: the extreme raw score times c (c may be negative)
        float mx = s[0][0];
        if (c >= 0.0f) {
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i >> 2][i & 3]);
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
        } else {
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fminf(mx, s[i >> 2][i & 3]);
            mx = fminf(mx, __shfl_xor(mx, 16));
            mx = fminf(mx, __shfl_xor(mx, 32));
        }
        // The reference maximum `top` only has to keep exp2() in range, the quotient does not depend
        // on it: it is moved (and the sums rescaled) only when some query of the wave would otherwise
        // exceed it by more than TAU, which after the first tile is rare.
        const float cand = mx * c;                       // finite: every tile holds at least one key
        if (__builtin_amdgcn_ballot_w64(cand > top + TAU) != 0) {
            const float new_top = fmaxf(top, cand);
            const float shrink = __builtin_amdgcn_exp2f(top - new_top);
            top = new_top;
            total *= shrink;
#pragma unroll
            for (int x = 0; x < 4 * HV; ++x) acc[x] *= shrink;
        }
        // probabilities exp2(c*s - top), rounded to bf16 for the second contraction
        u32x4 pf[2];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            pf[kb >> 1][(kb & 1) * 2] = pack_bf16(__builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][0], c, -top)),
                                                  __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][1], c, -top)));
            pf[kb >> 1][(kb & 1) * 2 + 1] = pack_bf16(__builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][2], c, -top)),
                                                      __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][3], c, -top)));
        }
        // O^T += V^T P^T: 4 blocks of 16 output columns, 2 k steps of 32 keys; a block of ones in
        // place of V^T yields the row sums of the rounded probabilities, for every lane of the query
#pragma unroll
        for (int h = 0; h < 2; ++h) total = mma(ones, pf[h], total);
        // The V fragments come by transposing reads issued as assembly (see xp_lds_tr.hpp), group by group
        // (one column block: 2 k steps, 4 reads), AHEAD groups in front of the MFMAs that use them; the
        // wait before a group's MFMAs leaves the reads of the younger groups outstanding.
        {
            constexpr int NG = 4 * HV, AHEAD = 3;
            FragHalves vf[NG][2];
            auto load_group = [&](auto gi_c) {
                constexpr int GI = decltype(gi_c)::value;
                const unsigned at = vx[GI % 4];
                vf[GI][0] = read_v(at, cur_c, std::integral_constant<int, GI / 4>{}, std::integral_constant<int, 0>{});
                vf[GI][1] = read_v(at, cur_c, std::integral_constant<int, GI / 4>{}, std::integral_constant<int, 1>{});
            };
            static_for<(AHEAD < NG ? AHEAD : NG)>([&](auto gi_c) { load_group(gi_c); });
            static_for<NG>([&](auto gi_c) {
                constexpr int GI = decltype(gi_c)::value;
                constexpr int YOUNGER = (NG - 1 - GI < AHEAD - 1 ? NG - 1 - GI : AHEAD - 1);
                lds_wait<4 * YOUNGER>();
                frag_tie(vf[GI][0]);
                frag_tie(vf[GI][1]);
#pragma unroll
                for (int h = 0; h < 2; ++h) acc[GI] = mma(frag_value(vf[GI][h]), pf[h], acc[GI]);
                __builtin_amdgcn_sched_barrier(0);       // or the scheduler collects the MFMAs behind the last wait
                if constexpr (GI + AHEAD < NG) load_group(std::integral_constant<int, GI + AHEAD>{});
            });
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(LPS * (D - 1)));
        wg_barrier();
    };
    // whole turns of the ring over the tiles that lie inside Lk, then what is left: fewer than NS such tiles and,
    // if Lk is no multiple of the tile, the ragged last one (NS tiles at most; the slots go on from 0)
    const int NF = Lk / BK;
    int t = 0;
    for (; t + NS <= NF; t += NS)
        static_for<NS>([&](auto u_c) { step(t + decltype(u_c)::value, std::false_type{}, u_c); });
    static_for<NS>([&](auto u_c) {
        constexpr int U = decltype(u_c)::value;
        if (t + U < NF) step(t + U, std::false_type{}, u_c);
        else if (t + U < NT) step(t + U, std::true_type{}, u_c);
    });
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));     // no load may outlive the wave

    const float inv = 1.0f / total[0];
    const int q = q0 + wave * 16 + r;
    if (q < p.Lq) {
        float *dst = p.O + b * p.strideO + (long long)q * p.ldo + 4 * g;
#pragma unroll
        for (int x = 0; x < 4 * HV; ++x) *(f32x4 *)(dst + 16 * x) = acc[x] * inv;
    }
}

// ------------------------------------------------------------------------------------ host side

AttnParams params_elements(const AttnProblem &q)
{
    AttnParams p;
    p.Q = (const char *)q.Q; p.K = (const char *)q.K; p.V = (const char *)q.V; p.O = (float *)q.O;
    p.Lq = (int)q.Lq; p.Lk = (int)q.Lk; p.d = (int)q.d; p.dv = (int)q.dv;
    p.ldq = q.ldq; p.ldk = q.ldk; p.ldv = q.ldv; p.ldo = q.ldo;
    p.strideQ = q.strideQ; p.strideK = q.strideK; p.strideV = q.strideV; p.strideO = q.strideO;
    p.scale = q.scale;
    return p;
}

bool general_can_run(const AttnProblem &q)
{
    return q.Lq <= 0x7fffffffLL && q.Lk <= 0x7fffffffLL && q.d <= 0x7fffffffLL && q.dv <= 0x7fffffffLL &&
           q.batch <= 65535 && (q.dv + 63) / 64 <= 65535;
}

hipError_t general_launch(const AttnProblem &q)
{
    const AttnParams p = params_elements(q);
    const dim3 grid((unsigned)q.Lq, (unsigned)q.batch, (unsigned)((q.dv + 63) / 64));
    if (q.in_type == XP_F32) hipLaunchKernelGGL(attn_general_kernel<float>, grid, dim3(64), 0, q.stream, p);
    else hipLaunchKernelGGL(attn_general_kernel<unsigned short>, grid, dim3(64), 0, q.stream, p);
    return hipGetLastError();
}

template <int HV>
bool mfma_can_run(const AttnProblem &q)
{
    if (q.in_type != XP_BF16 || q.d != HD * HV || q.dv != HD * HV) return false;
    if (q.scale == 0.0f) return false;                   // the kernel masks absent keys by an infinite raw score times the scale
    if (q.batch > 65535 || q.Lq > 0x3fffffffLL || q.Lk > 0x3fffffffLL) return false;
    const void *ptrs[3] = {q.Q, q.K, q.V};
    const int64_t lds_[3] = {q.ldq, q.ldk, q.ldv}, strides[3] = {q.strideQ, q.strideK, q.strideV};
    const int64_t rows[3] = {q.Lq, q.Lk, q.Lk};
    for (int i = 0; i < 3; ++i) {
        if (((uintptr_t)ptrs[i] % 16) != 0 || (lds_[i] * 2) % 16 != 0 || (strides[i] * 2) % 16 != 0) return false;
        if ((rows[i] + 4 * BK) * lds_[i] * 2 >= 0x7fffffffLL) return false;  // 32-bit byte offsets, prefetch past the end included
    }
    if (((uintptr_t)q.O % 16) != 0 || (q.ldo * 4) % 16 != 0 || (q.strideO * 4) % 16 != 0) return false;
    return true;
}

template <int D, int HV, int NW>
hipError_t mfma_launch(const AttnProblem &q)
{
    AttnParams p = params_elements(q);
    p.ldq *= 2; p.ldk *= 2; p.ldv *= 2;                  // bytes
    p.strideQ *= 2; p.strideK *= 2; p.strideV *= 2;
    const dim3 grid((unsigned)((q.Lq + 16 * NW - 1) / (16 * NW)), (unsigned)q.batch);
    hipLaunchKernelGGL((attn_mfma_kernel<D, HV, NW>), grid, dim3(64 * NW), 0, q.stream, p);
    return hipGetLastError();
}

const AttnVariant kGeneral = {"general attention one wave per query valu", general_can_run, general_launch};
const AttnVariant kMfma64d1 = {"bf16 attention head 64, 64 queries x 64-key steps, prefetch 1, waves 4x1 mfma16", mfma_can_run<1>,
                               mfma_launch<1, 1, 4>};
const AttnVariant kMfma64d2 = {"bf16 attention head 64, 64 queries x 64-key steps, prefetch 2, waves 4x1 mfma16", mfma_can_run<1>,
                               mfma_launch<2, 1, 4>};
const AttnVariant kMfma128d1 = {"bf16 attention head 128, 64 queries x 64-key steps, prefetch 1, waves 4x1 mfma16", mfma_can_run<2>,
                                mfma_launch<1, 2, 4>};
const AttnVariant kMfma128d2 = {"bf16 attention head 128, 64 queries x 64-key steps, prefetch 2, waves 4x1 mfma16", mfma_can_run<2>,
                                mfma_launch<2, 2, 4>};
// Eight waves per workgroup pay when there are enough such workgroups: two per compute unit at head size 64, one at
// head size 128 (swept under sustained load, TFLOP/s with 8 / 4 waves: head 64 -- 32 x 2048^2 732 / 667, 192 x 512^2
// 550 / 510, but 96 x 512^2 (384 workgroups of 128 queries) 423 / 460 and 48 x 1024^2 528 / 560; head 128 --
// 32 x 2048^2 891 / 740, 96 x 512^2 (384) 513 / 479, 8 x 4096^2 (256) 856 / 778)
bool w8_worthwhile_64(const AttnProblem &q) { return q.batch * ((q.Lq + 127) / 128) >= 512; }
bool w8_worthwhile_128(const AttnProblem &q) { return q.batch * ((q.Lq + 127) / 128) >= 256; }
const AttnVariant kMfma64w8 = {"bf16 attention head 64, 128 queries x 64-key steps, prefetch 1, waves 8x1 mfma16", mfma_can_run<1>,
                               mfma_launch<1, 1, 8>, w8_worthwhile_64};
const AttnVariant kMfma128w8 = {"bf16 attention head 128, 128 queries x 64-key steps, prefetch 1, waves 8x1 mfma16", mfma_can_run<2>,
                                mfma_launch<1, 2, 8>, w8_worthwhile_128};
// swept on the 96 x 512 x 512 x 64 workload: a prefetch distance of 1 is as fast as 2 (the step is bound
// by its own dependency chain, not by load latency) and leaves more LDS free; 3 is slower
const AttnVariant *const kBf16Table[] = {&kGeneral, &kMfma64d2, &kMfma64d1, &kMfma128d2, &kMfma128d1, &kMfma64w8, &kMfma128w8};   // the last that can run is the default

}  // namespace

int attn_num_variants(xp_dtype in_type) { return in_type == XP_BF16 ? 7 : (in_type == XP_F32 ? 1 : 0); }

const AttnVariant *attn_variant(xp_dtype in_type, int idx)
{
    if (idx < 0 || idx >= attn_num_variants(in_type)) return nullptr;
    return in_type == XP_BF16 ? kBf16Table[idx] : &kGeneral;
}

}  // namespace xp
