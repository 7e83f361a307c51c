// Multi-scale deformable attention (Table 5, "Deformable Attention"; the paper's Section 6 singles it
// out as the hardest operator of its benchmark): every (query, head) gathers levels x points bilinear
// samples from the value maps and adds them up with its attention weights.  There is no contraction
// and no reuse between queries that a tile could exploit -- the sampling positions are data -- so
// the kernel is a gather: one lane per (query, head, 16-byte channel chunk), the positions and
// weights of a (query, head) read once (the lanes of its chunks share the addresses), the four
// corner pixels fetched as 16-byte chunks through the caches, fp32 accumulation in registers, one
// streaming store.  Lanes next to each other cover the chunks of one head, then the heads of one
// query, so that a wavefront's corner fetches fall on whole 64..128-byte pixel rows.
#include "xp_internal.hpp"

namespace xp {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int MAX_LEVELS = 16;

struct DeformParams {
    const void *value;
    const float *loc, *wgt;
    void *out;
    long long units;                     // batch * Lq * heads * (d / EPC)
    long long S;                         // pixels of all levels together
    int Lq, heads, d, levels, points;
    int H[MAX_LEVELS], W[MAX_LEVELS];
    long long start[MAX_LEVELS];         // first pixel of a level
};

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));      // round to nearest even
}

// EPC channels of one pixel: fetched as raw words, widened to fp32 later, so that the loads of
// several sampling points can be in flight before the first is consumed
template <bool BF16, int EPC> struct Pixel {
    u32x4 w;
    __device__ __forceinline__ void fetch(const char *at)
    {
        if constexpr (EPC == 1) {
            if constexpr (BF16) w[0] = (unsigned)*(const unsigned short *)at << 16;
            else w[0] = *(const unsigned *)at;
        } else {
            w = *(const u32x4 *)at;
        }
    }
    // a corner outside the map is zero whatever the word fetched from the clamped address holds
    __device__ __forceinline__ void keep_if(bool inside)
    {
#pragma unroll
        for (int i = 0; i < (EPC == 1 ? 1 : 4); ++i) w[i] = inside ? w[i] : 0u;
    }
    __device__ __forceinline__ void accumulate(float weight, float (&acc)[EPC]) const
    {
        if constexpr (EPC == 1) {
            acc[0] = __builtin_fmaf(weight, __uint_as_float(w[0]), acc[0]);
        } else if constexpr (BF16) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] = __builtin_fmaf(weight, __uint_as_float(w[i] << 16), acc[2 * i]);
                acc[2 * i + 1] = __builtin_fmaf(weight, __uint_as_float(w[i] & 0xffff0000u), acc[2 * i + 1]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(weight, __uint_as_float(w[i]), acc[i]);
        }
    }
};

constexpr int PU = 4;      // sampling points handled together: 16 corner fetches in flight per lane

// PU sampling points of one (query, head) on one level.  `map` is the address of this lane's channels
// in pixel (0,0) of the level (global memory or LDS), `pitch` the bytes from one pixel to the next;
// (lx, ly) the normalised position, a the attention weight, live[j] false for a padding slot.
// Branch-free per point: positions outside (or NaN) keep a zero weight and fetch pixel (0,0); corners
// outside are fetched from the clamped address and zeroed afterwards.  H, W >= 1.
template <bool BF16, int EPC>
__device__ __forceinline__ void sample_points(const char *map, long long pitch, int H, int W, const float (&lx)[PU],
                                              const float (&ly)[PU], const float (&aw)[PU], const bool (&live)[PU],
                                              float (&acc)[EPC])
{
    Pixel<BF16, EPC> px[PU][4];
    float cw[PU][4];
    bool in[PU][4];
#pragma unroll
    for (int j = 0; j < PU; ++j) {
        // normalised -> pixel coordinates, pixel centres at half-integers
        float x = __builtin_fmaf(lx[j], (float)W, -0.5f), y = __builtin_fmaf(ly[j], (float)H, -0.5f);
        // the comparisons are false for NaN too: such a point, like one a pixel or more outside, adds nothing
        const bool ok = live[j] && x > -1.0f && x < (float)W && y > -1.0f && y < (float)H;
        x = ok ? x : 0.0f;
        y = ok ? y : 0.0f;
        const float a = ok ? aw[j] : 0.0f;
        const float xf = __builtin_floorf(x), yf = __builtin_floorf(y);
        const int x0 = (int)xf, y0 = (int)yf;             // in [-1, W-1], [-1, H-1]
        const float fx = x - xf, fy = y - yf;
        const bool left = x0 >= 0, right = x0 + 1 < W, top = y0 >= 0, bottom = y0 + 1 < H;
        const int xl = left ? x0 : 0, xr = right ? x0 + 1 : W - 1, yt = top ? y0 : 0, yb = bottom ? y0 + 1 : H - 1;
        cw[j][0] = a * (1.0f - fy) * (1.0f - fx); in[j][0] = ok && top && left;
        cw[j][1] = a * (1.0f - fy) * fx;          in[j][1] = ok && top && right;
        cw[j][2] = a * fy * (1.0f - fx);          in[j][2] = ok && bottom && left;
        cw[j][3] = a * fy * fx;                   in[j][3] = ok && bottom && right;
        px[j][0].fetch(map + ((long long)yt * W + xl) * pitch);
        px[j][1].fetch(map + ((long long)yt * W + xr) * pitch);
        px[j][2].fetch(map + ((long long)yb * W + xl) * pitch);
        px[j][3].fetch(map + ((long long)yb * W + xr) * pitch);
    }
#pragma unroll
    for (int j = 0; j < PU; ++j)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            px[j][k].keep_if(in[j][k]);
            px[j][k].accumulate(cw[j][k], acc);
        }
}

// Any number of points: positions and weights read one point at a time.
template <bool BF16, int EPC>
__device__ __forceinline__ void sample_level(const char *map, long long pitch, int H, int W, const float *loc, const float *wgt,
                                             int points, float (&acc)[EPC])
{
    for (int pt0 = 0; pt0 < points; pt0 += PU) {
        float lx[PU], ly[PU], aw[PU];
        bool live[PU];
#pragma unroll
        for (int j = 0; j < PU; ++j) {
            live[j] = pt0 + j < points;
            const int pt = live[j] ? pt0 + j : points - 1;
            const f32x2 xy = *(const f32x2 *)(loc + 2 * pt);
            lx[j] = xy[0];
            ly[j] = xy[1];
            aw[j] = wgt[pt];
        }
        sample_points<BF16, EPC>(map, pitch, H, W, lx, ly, aw, live, acc);
    }
}

// Four points per level (the usual configuration): the positions and weights of a level are 32 + 16
// contiguous bytes, read as three 16-byte words -- and read one level ahead of their use, so that
// their latency is covered by the gathers of the level before.
struct LevelPoints {
    u32x4 xy01, xy23, a;
    __device__ __forceinline__ void load(const float *loc, const float *wgt)
    {
        xy01 = __builtin_nontemporal_load((const u32x4 *)loc);
        xy23 = __builtin_nontemporal_load((const u32x4 *)loc + 1);
        a = __builtin_nontemporal_load((const u32x4 *)wgt);
    }
};
template <bool BF16, int EPC>
__device__ __forceinline__ void sample_level4(const char *map, long long pitch, int H, int W, const LevelPoints &s,
                                              float (&acc)[EPC])
{
    const float lx[PU] = {__uint_as_float(s.xy01[0]), __uint_as_float(s.xy01[2]), __uint_as_float(s.xy23[0]), __uint_as_float(s.xy23[2])};
    const float ly[PU] = {__uint_as_float(s.xy01[1]), __uint_as_float(s.xy01[3]), __uint_as_float(s.xy23[1]), __uint_as_float(s.xy23[3])};
    const float aw[PU] = {__uint_as_float(s.a[0]), __uint_as_float(s.a[1]), __uint_as_float(s.a[2]), __uint_as_float(s.a[3])};
    const bool live[PU] = {true, true, true, true};
    sample_points<BF16, EPC>(map, pitch, H, W, lx, ly, aw, live, acc);
}

// Four points per level and four lanes per (query, head) -- 32 bf16 or 16 fp32 channels a head: the
// arithmetic on the positions, a third of the instructions when every lane does it for every point,
// is shared out.  Lane j of the quad works out point j alone (clamped corner offsets, corner weights
// with the corners outside the map already at zero), then the quad exchanges the results with
// quad-broadcast moves.  A point wholly outside (or NaN) fetches pixel (0,0) with zero weights and has
// the fetched words blanked, so that nothing a caller left in that pixel can reach the sum.
template <int J> __device__ __forceinline__ unsigned quad_bcast(unsigned v)
{
    // (the source as the fallback value too: every lane of a quad permutation has a source, and a constant there
    // would cost a register initialisation per broadcast)
    return (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, J * 0x55, 0xf, 0xf, true);      // quad_perm [J,J,J,J]
}
template <int J> __device__ __forceinline__ float quad_bcast(float v) { return __uint_as_float(quad_bcast<J>(__float_as_uint(v))); }

template <bool BF16, int EPC> struct QuadSampler {
    Pixel<BF16, EPC> px[4][4];
    float cw[4][4];
    unsigned ok[4];

    // the lane's own point: corner offsets in bytes from pixel (0,0) of the level (they fit 32 bits)
    unsigned own_off[4];
    float own_cw[4];
    unsigned own_ok;
    // bf16 values: the corner weights as two bf16 terms each (w = hi + lo up to 2^-18 w), packed in
    // corner pairs {0,1} and {2,3} -- the A operand of the matrix-core sum below
    unsigned own_hi[2], own_lo[2];
    unsigned wa[4][2];
    __device__ __forceinline__ void prepare(unsigned pitch, int H, int W, f32x2 xy, float aw)
    {
        float x = __builtin_fmaf(xy[0], (float)W, -0.5f), y = __builtin_fmaf(xy[1], (float)H, -0.5f);
        const bool inside = x > -1.0f && x < (float)W && y > -1.0f && y < (float)H;      // false for NaN too
        x = inside ? x : 0.0f;
        y = inside ? y : 0.0f;
        const float a = inside ? aw : 0.0f;
        const float xf = __builtin_floorf(x), yf = __builtin_floorf(y);
        const int x0 = (int)xf, y0 = (int)yf;
        const float fx = x - xf, fy = y - yf;
        const bool left = x0 >= 0, right = x0 + 1 < W, top = y0 >= 0, bottom = y0 + 1 < H;
        const int xl = left ? x0 : 0, xr = right ? x0 + 1 : W - 1, yt = top ? y0 : 0, yb = bottom ? y0 + 1 : H - 1;
        own_cw[0] = top && left ? a * (1.0f - fy) * (1.0f - fx) : 0.0f;
        own_cw[1] = top && right ? a * (1.0f - fy) * fx : 0.0f;
        own_cw[2] = bottom && left ? a * fy * (1.0f - fx) : 0.0f;
        own_cw[3] = bottom && right ? a * fy * fx : 0.0f;
        own_off[0] = (unsigned)(yt * W + xl) * pitch;
        own_off[1] = (unsigned)(yt * W + xr) * pitch;
        own_off[2] = (unsigned)(yb * W + xl) * pitch;
        own_off[3] = (unsigned)(yb * W + xr) * pitch;
        own_ok = inside ? 1u : 0u;
        if constexpr (BF16) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                own_hi[h] = pack_bf16(own_cw[2 * h], own_cw[2 * h + 1]);
                own_lo[h] = pack_bf16(own_cw[2 * h] - __uint_as_float(own_hi[h] << 16),
                                      own_cw[2 * h + 1] - __uint_as_float(own_hi[h] & 0xffff0000u));
            }
        }
    }
    template <int J> __device__ __forceinline__ void fetch_point(const char *map)
    {
        ok[J] = quad_bcast<J>(own_ok);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if constexpr (!BF16) cw[J][k] = quad_bcast<J>(own_cw[k]);
            px[J][k].fetch(map + quad_bcast<J>(own_off[k]));
        }
        if constexpr (BF16) {
            // odd lanes of the quad carry the low terms, even lanes the high terms (rows 0 and 1 of the
            // matrix product are used, rows 2 and 3 repeat them and are ignored)
            const bool low = threadIdx.x & 1;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const unsigned hi = quad_bcast<J>(own_hi[h]), lo = quad_bcast<J>(own_lo[h]);
                wa[J][h] = low ? lo : hi;
            }
        }
    }
    __device__ __forceinline__ void fetch(const char *map)
    {
        fetch_point<0>(map); fetch_point<1>(map); fetch_point<2>(map); fetch_point<3>(map);
    }
    // bf16 values: the weighted sum of the four corners on the matrix cores.  v_mfma_f32_4x4x4_16B_bf16
    // multiplies sixteen independent 4x4 blocks, one per lane quad: D[i][j] = sum_k A[i][k] B[k][j] with
    // row i of A taken from lane i of the quad, column j of B and of D held by lane j.  Here k runs over
    // the corners, column j is channel e of lane j's chunk, and the rows are the high and the low bf16
    // terms of the corner weights: rows 0 and 1 of D add up to the fp32-weighted sum.  Per point that is
    // 8 matrix instructions and 16 byte permutes (which also blank a point outside the map) in place
    // of 32 widenings and 32 FMAs.
    __device__ __forceinline__ void accumulate_mfma(f32x4 (&accm)[8]) const
    {
        static_assert(BF16 && EPC == 8, "bf16 chunks of eight channels");
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned sel_even = ok[j] ? 0x05040100u : 0x0c0c0c0cu, sel_odd = ok[j] ? 0x07060302u : 0x0c0c0c0cu;
            const u32x2 aw = {wa[j][0], wa[j][1]};
            const s16x4 a = __builtin_bit_cast(s16x4, aw);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned sel = (e & 1) ? sel_odd : sel_even;
                const u32x2 bw = {__builtin_amdgcn_perm(px[j][1].w[e >> 1], px[j][0].w[e >> 1], sel),
                                  __builtin_amdgcn_perm(px[j][3].w[e >> 1], px[j][2].w[e >> 1], sel)};
                accm[e] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, __builtin_bit_cast(s16x4, bw), accm[e], 0, 0, 0);
            }
        }
    }
    __device__ __forceinline__ void accumulate(float (&acc)[EPC]) const
    {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (BF16) {
                // byte selectors of the two widenings (low half -> bits 31..16, high half kept), all-zero for a blanked point
                const unsigned sel_lo = ok[j] ? 0x01000c0cu : 0x0c0c0c0cu, sel_hi = ok[j] ? 0x03020c0cu : 0x0c0c0c0cu;
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const unsigned w = px[j][k].w[i];
                        acc[2 * i] = __builtin_fmaf(cw[j][k], __uint_as_float(__builtin_amdgcn_perm(0u, w, sel_lo)), acc[2 * i]);
                        acc[2 * i + 1] = __builtin_fmaf(cw[j][k], __uint_as_float(__builtin_amdgcn_perm(0u, w, sel_hi)), acc[2 * i + 1]);
                    }
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    Pixel<BF16, EPC> v = px[j][k];
                    v.keep_if(ok[j] != 0);
                    v.accumulate(cw[j][k], acc);
                }
            }
        }
    }
};

// o: element index of the first of EPC output channels
template <bool OUT_BF16, int EPC> __device__ __forceinline__ void store_out(void *out, long long o, const float (&acc)[EPC])
{
    if constexpr (EPC == 1) {
        if constexpr (OUT_BF16) ((unsigned short *)out)[o] = (unsigned short)pack_bf16(acc[0], 0.0f);
        else ((float *)out)[o] = acc[0];
    } else if constexpr (OUT_BF16) {
        unsigned w[EPC / 2];
#pragma unroll
        for (int i = 0; i < EPC / 2; ++i) w[i] = pack_bf16(acc[2 * i], acc[2 * i + 1]);
        if constexpr (EPC == 8) __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, (u32x4 *)((unsigned short *)out + o));
        else __builtin_nontemporal_store(u32x2{w[0], w[1]}, (u32x2 *)((unsigned short *)out + o));
    } else {
#pragma unroll
        for (int i = 0; i < EPC; i += 4)
            __builtin_nontemporal_store(u32x4{__float_as_uint(acc[i]), __float_as_uint(acc[i + 1]), __float_as_uint(acc[i + 2]),
                                              __float_as_uint(acc[i + 3])}, (u32x4 *)((float *)out + o + i));
    }
}

// General kernel: one lane per (query, head, chunk), every corner from global memory.
// MODE: how the positions and weights are read -- ANY number of points, FOUR points a level as 16-byte
// words, or QUAD: four points a level and four lanes a head, each lane preparing one point.
enum { ANY = 0, FOUR = 1, QUAD = 2 };

template <bool BF16, bool OUT_BF16, int EPC, int MODE> __global__ __launch_bounds__(256) void deform_kernel(DeformParams p)
{
    constexpr int ES = BF16 ? 2 : 4;
    const long long unit = (long long)xcd_chunked(blockIdx.x, gridDim.x) * 256 + threadIdx.x;
    if (unit >= p.units) return;
    const int chunks = p.d / EPC;
    const long long nqm = unit / chunks;                         // (n * Lq + q) * heads + m
    const int c0 = (int)(unit - nqm * chunks) * EPC;
    const int m = (int)(nqm % p.heads);
    const long long n = nqm / p.heads / p.Lq;
    const long long pixel_stride = (long long)p.heads * p.d;     // elements from one pixel to the next
    const long long base = n * p.S * pixel_stride + (long long)m * p.d + c0;

    float acc[EPC];
#pragma unroll
    for (int i = 0; i < EPC; ++i) acc[i] = 0.0f;
    f32x4 accm[8];                                               // QUAD with bf16 values: see accumulate_mfma
#pragma unroll
    for (int i = 0; i < 8; ++i) accm[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const long long at0 = nqm * p.levels * p.points;
    LevelPoints ahead;
    if constexpr (MODE == FOUR) if (p.levels > 0) ahead.load(p.loc + 2 * at0, p.wgt + at0);
    const int lane_pt = threadIdx.x & 3;                         // QUAD: the point this lane prepares
    f32x2 xy_ahead = {0.0f, 0.0f};
    float a_ahead = 0.0f;
    if constexpr (MODE == QUAD) if (p.levels > 0) {
        xy_ahead = __builtin_nontemporal_load((const f32x2 *)(p.loc + 2 * (at0 + lane_pt)));
        a_ahead = __builtin_nontemporal_load(p.wgt + at0 + lane_pt);
    }
    for (int l = 0; l < p.levels; ++l) {
        const int H = p.H[l], W = p.W[l];
        const long long at = at0 + (long long)l * p.points;
        const char *map = (const char *)p.value + (base + p.start[l] * pixel_stride) * ES;
        if constexpr (MODE == QUAD) {
            const f32x2 xy = xy_ahead;
            const float aw = a_ahead;
            if (l + 1 < p.levels) {
                xy_ahead = __builtin_nontemporal_load((const f32x2 *)(p.loc + 2 * (at + 4 + lane_pt)));
                a_ahead = __builtin_nontemporal_load(p.wgt + at + 4 + lane_pt);
            }
            if (H == 0 || W == 0) continue;
            QuadSampler<BF16, EPC> qs;
            qs.prepare((unsigned)(pixel_stride * ES), H, W, xy, aw);
            qs.fetch(map);
            if constexpr (BF16) qs.accumulate_mfma(accm);
            else qs.accumulate(acc);
        } else if constexpr (MODE == FOUR) {
            const LevelPoints now = ahead;
            if (l + 1 < p.levels) ahead.load(p.loc + 2 * (at + 4), p.wgt + at + 4);
            if (H == 0 || W == 0) continue;                      // an empty level has nothing to sample
            sample_level4<BF16, EPC>(map, pixel_stride * ES, H, W, now, acc);
        } else {
            if (H == 0 || W == 0) continue;
            sample_level<BF16, EPC>(map, pixel_stride * ES, H, W, p.loc + 2 * at, p.wgt + at, p.points, acc);
        }
    }
    if constexpr (MODE == QUAD && BF16) {
#pragma unroll
        for (int i = 0; i < EPC; ++i) acc[i] = accm[i][0] + accm[i][1];
    }
    store_out<OUT_BF16, EPC>(p.out, nqm * p.d + c0, acc);
}

// Kernel with the small levels in LDS.  In an encoder layer every pixel of the coarse levels is
// sampled by hundreds of queries, but a compute unit's 32 KB vector cache, shared by all the heads in
// flight, keeps few of them: the general kernel sends three of four corner fetches on to the L2 and
// runs at the L2's request rate.  Here a workgroup serves one (image, head) and a block of queries:
// it first copies that head's channels of the chosen levels (the smallest ones, as many as fit) into
// LDS, then its lanes take the corners of those levels from LDS and only the remaining levels'
// from global memory.  Lane layout: CH = d/EPC lanes per query, 512/CH queries per pass.
struct LdsPlan {
    int lds_off[MAX_LEVELS];             // byte offset of a staged level, -1: sampled from global memory
    int queries_per_wg;
    unsigned qblocks, items;             // query blocks per (image, head); workgroups with work
    int first_global;                    // first non-empty level that is not staged, -1 if there is none
};
constexpr int LDS_THREADS = 512;

template <bool BF16, bool OUT_BF16, int MODE> __global__ __launch_bounds__(LDS_THREADS) void deform_lds_kernel(DeformParams p, LdsPlan plan)
{
    constexpr int EPC = BF16 ? 8 : 4, ES = BF16 ? 2 : 4;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const unsigned item = xcd_chunked(blockIdx.x, gridDim.x);    // (image, head, query block), query block fastest
    if (item >= plan.items) return;
    const int qblock = item % plan.qblocks;
    const int m = (item / plan.qblocks) % p.heads;
    const long long n = item / plan.qblocks / p.heads;
    const int CH = p.d / EPC;                                    // divides LDS_THREADS
    const int PB = p.d * ES;                                     // bytes of one pixel of one head
    const long long pixel_stride = (long long)p.heads * p.d;
    const long long head_base = n * p.S * pixel_stride + (long long)m * p.d;

    for (int l = 0; l < p.levels; ++l) {
        if (plan.lds_off[l] < 0) continue;
        const int chunks = p.H[l] * p.W[l] * CH;
        const char *src = (const char *)p.value + (head_base + p.start[l] * pixel_stride) * ES;
        for (int i = tid; i < chunks; i += LDS_THREADS) {
            const int px = i / CH, c = i - px * CH;
            *(u32x4 *)(lds + plan.lds_off[l] + px * PB + c * 16) = *(const u32x4 *)(src + (long long)px * pixel_stride * ES + c * 16);
        }
    }
    __syncthreads();

    const int c = tid % CH;
    const int q_first = qblock * plan.queries_per_wg;
    const int q_end = min(p.Lq, q_first + plan.queries_per_wg);
    if constexpr (MODE == QUAD) {
        // At most four levels, four points each, lane c of a head prepares point c.  Loads return in
        // order, so the sequence of a pass is: the positions and weights of the *next* pass (used only
        // then), the gathers of the one level that lives in global memory, then -- while those are in
        // flight -- the staged levels out of LDS, and last the sum over the global level's corners.
        constexpr int ML = 4;
        const int stride = LDS_THREADS / CH;
        const int g = plan.first_global;
        f32x2 xy_next[ML];
        float a_next[ML];
        auto load_points = [&](int q, f32x2 (&xy)[ML], float (&a)[ML]) {
            const long long at0 = ((n * p.Lq + q) * p.heads + m) * (long long)p.levels * 4 + c;
#pragma unroll
            for (int l = 0; l < ML; ++l) {
                xy[l] = f32x2{0.0f, 0.0f};
                a[l] = 0.0f;
                if (l < p.levels) {
                    xy[l] = __builtin_nontemporal_load((const f32x2 *)(p.loc + 2 * (at0 + 4 * l)));
                    a[l] = __builtin_nontemporal_load(p.wgt + at0 + 4 * l);
                }
            }
        };
        int q = q_first + tid / CH;
        if (q < q_end) load_points(q, xy_next, a_next);
        for (; q < q_end; q += stride) {
            f32x2 xy[ML];
            float a[ML];
#pragma unroll
            for (int l = 0; l < ML; ++l) { xy[l] = xy_next[l]; a[l] = a_next[l]; }
            if (q + stride < q_end) load_points(q + stride, xy_next, a_next);
            float acc[EPC];
#pragma unroll
            for (int i = 0; i < EPC; ++i) acc[i] = 0.0f;
            f32x4 accm[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) accm[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            QuadSampler<BF16, EPC> qg;
#pragma unroll
            for (int l = 0; l < ML; ++l)
                if (l == g) {
                    qg.prepare((unsigned)(pixel_stride * ES), p.H[l], p.W[l], xy[l], a[l]);
                    qg.fetch((const char *)p.value + (head_base + p.start[l] * pixel_stride) * ES + c * 16);
                }
#pragma unroll
            for (int l = 0; l < ML; ++l) {
                if (l >= p.levels || l == g) continue;
                const int H = p.H[l], W = p.W[l];
                if (H == 0 || W == 0) continue;
                const bool staged = plan.lds_off[l] >= 0;
                QuadSampler<BF16, EPC> qs;
                qs.prepare(staged ? (unsigned)PB : (unsigned)(pixel_stride * ES), H, W, xy[l], a[l]);
                if (staged) qs.fetch(lds + plan.lds_off[l] + c * 16);
                else qs.fetch((const char *)p.value + (head_base + p.start[l] * pixel_stride) * ES + c * 16);
                if constexpr (BF16) qs.accumulate_mfma(accm);
                else qs.accumulate(acc);
            }
            if (g >= 0) {
                if constexpr (BF16) qg.accumulate_mfma(accm);
                else qg.accumulate(acc);
            }
            if constexpr (BF16) {
#pragma unroll
                for (int i = 0; i < EPC; ++i) acc[i] = accm[i][0] + accm[i][1];
            }
            store_out<OUT_BF16, EPC>(p.out, ((n * p.Lq + q) * p.heads + m) * p.d + c * EPC, acc);
        }
        return;
    }
    for (int q = q_first + tid / CH; q < q_end; q += LDS_THREADS / CH) {
        const long long nqm = (n * p.Lq + q) * p.heads + m;
        float acc[EPC];
#pragma unroll
        for (int i = 0; i < EPC; ++i) acc[i] = 0.0f;
        const long long at0 = nqm * p.levels * p.points;
        LevelPoints ahead;
        if constexpr (MODE == FOUR) ahead.load(p.loc + 2 * at0, p.wgt + at0);
        for (int l = 0; l < p.levels; ++l) {
            const int H = p.H[l], W = p.W[l];
            const long long at = at0 + (long long)l * p.points;
            const bool staged = plan.lds_off[l] >= 0;
            const char *global_map = (const char *)p.value + (head_base + p.start[l] * pixel_stride) * ES + c * 16;
            const char *lds_map = lds + (staged ? plan.lds_off[l] : 0) + c * 16;
            if constexpr (MODE == FOUR) {
                const LevelPoints now = ahead;
                if (l + 1 < p.levels) ahead.load(p.loc + 2 * (at + 4), p.wgt + at + 4);
                if (H == 0 || W == 0) continue;
                if (staged) sample_level4<BF16, EPC>(lds_map, PB, H, W, now, acc);
                else sample_level4<BF16, EPC>(global_map, pixel_stride * ES, H, W, now, acc);
            } else {
                if (H == 0 || W == 0) continue;
                if (staged) sample_level<BF16, EPC>(lds_map, PB, H, W, p.loc + 2 * at, p.wgt + at, p.points, acc);
                else sample_level<BF16, EPC>(global_map, pixel_stride * ES, H, W, p.loc + 2 * at, p.wgt + at, p.points, acc);
            }
        }
        store_out<OUT_BF16, EPC>(p.out, nqm * p.d + c * EPC, acc);
    }
}

// FOUR: four points per level and positions / weights on 16-byte boundaries (the three-word reads);
// QUAD: four points, four 16-byte chunks a head, every level's byte offsets inside 32 bits
int read_mode(const DeformParams &p, int epc, int es)
{
    if (p.points != 4) return ANY;
    if (p.d == 4 * epc) {
        bool fits = true;
        for (int l = 0; l < p.levels; ++l)
            fits = fits && (long double)p.H[l] * p.W[l] * p.heads * p.d * es < 4.0e9L && (long long)p.H[l] * p.W[l] < (1LL << 31);
        if (fits) return QUAD;
    }
    return (uintptr_t)p.loc % 16 == 0 && (uintptr_t)p.wgt % 16 == 0 ? FOUR : ANY;
}

template <bool BF16, bool OUT_BF16, int EPC> xp_status launch(const DeformParams &p, hipStream_t stream)
{
    const long long blocks = ((p.units + 255) / 256 + 7) / 8 * 8;          // a multiple of 8: see xcd_chunked
    if (blocks > 0x7fffffffLL) return XP_ERR_SHAPE;
    const int mode = EPC == 1 ? ANY : read_mode(p, EPC, BF16 ? 2 : 4);
    if constexpr (EPC > 1) {
        if (mode == QUAD) hipLaunchKernelGGL((deform_kernel<BF16, OUT_BF16, EPC, QUAD>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
        else if (mode == FOUR) hipLaunchKernelGGL((deform_kernel<BF16, OUT_BF16, EPC, FOUR>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    }
    if (mode == ANY) hipLaunchKernelGGL((deform_kernel<BF16, OUT_BF16, EPC, ANY>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    return hipGetLastError() == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

constexpr int LDS_BUDGET = 96 * 1024;     // staged bytes per workgroup at most (one workgroup per compute unit above 80 KB)
constexpr int NUM_CUS = 256;

// Decides whether staging pays and which levels are staged; false: use the general kernel.
bool plan_lds(const DeformParams &p, long long batch, int es, int epc, LdsPlan &plan, int &lds_bytes, dim3 &grid)
{
    if (p.d % epc || LDS_THREADS % (p.d / epc) || p.points == 0 || p.levels == 0) return false;
    if (p.Lq > (1 << 30)) return false;
    const int PB = p.d * es;
    // levels by size, smallest first, while they fit
    int order[MAX_LEVELS];
    for (int l = 0; l < p.levels; ++l) order[l] = l;
    for (int i = 1; i < p.levels; ++i)
        for (int j = i; j > 0 && (long long)p.H[order[j]] * p.W[order[j]] < (long long)p.H[order[j - 1]] * p.W[order[j - 1]]; --j) {
            const int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t;
        }
    for (int l = 0; l < p.levels; ++l) plan.lds_off[l] = -1;
    long long staged = 0;
    int nstaged = 0;
    for (int i = 0; i < p.levels; ++i) {
        const int l = order[i];
        const long long bytes = (long long)p.H[l] * p.W[l] * PB;
        if (bytes == 0) continue;
        if (staged + bytes > LDS_BUDGET) break;
        plan.lds_off[l] = (int)staged;
        staged += bytes;
        ++nstaged;
    }
    if (nstaged == 0) return false;
    // query blocks: about one workgroup per compute unit and (image, head) rounds, each with enough
    // queries that the copy into LDS is small beside what is then gathered from it
    const long long pairs = batch * p.heads;
    long long qblocks = (NUM_CUS + pairs - 1) / pairs;
    if (qblocks > p.Lq) qblocks = p.Lq;
    const long long qpw = (p.Lq + qblocks - 1) / qblocks;
    const long long gathered = qpw * nstaged * p.points * 4 * PB;
    if (staged * 4 > gathered) return false;
    plan.first_global = -1;
    for (int l = p.levels - 1; l >= 0; --l)
        if (plan.lds_off[l] < 0 && p.H[l] > 0 && p.W[l] > 0) plan.first_global = l;
    plan.queries_per_wg = (int)qpw;
    plan.qblocks = (unsigned)((p.Lq + qpw - 1) / qpw);
    const long long items = pairs * plan.qblocks;
    if (items > 0x7ffffff0LL) return false;
    plan.items = (unsigned)items;
    lds_bytes = (int)staged;
    grid = dim3((unsigned)((items + 7) / 8 * 8));
    return true;
}

template <bool BF16, bool OUT_BF16> xp_status launch_lds(const DeformParams &p, const LdsPlan &plan, int lds_bytes, dim3 grid,
                                                         hipStream_t stream)
{
    int mode = read_mode(p, BF16 ? 8 : 4, BF16 ? 2 : 4);
    if (mode == QUAD && p.levels > 4)            // that kernel keeps a pass's positions of all levels in registers
        mode = (uintptr_t)p.loc % 16 == 0 && (uintptr_t)p.wgt % 16 == 0 ? FOUR : ANY;
    auto kernel = mode == QUAD ? deform_lds_kernel<BF16, OUT_BF16, QUAD>
                : mode == FOUR ? deform_lds_kernel<BF16, OUT_BF16, FOUR> : deform_lds_kernel<BF16, OUT_BF16, ANY>;
    if (lds_bytes > 48 * 1024 &&
        hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
        return XP_ERR_LAUNCH;
    hipLaunchKernelGGL(kernel, grid, dim3(LDS_THREADS), lds_bytes, stream, p, plan);
    return hipGetLastError() == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

}  // namespace
}  // namespace xp

extern "C" xp_status xp_deformable_attention(int64_t batch, int64_t Lq, int64_t heads, int64_t d, int64_t levels, int64_t points,
                                             const void *value, xp_dtype v_type, const int64_t *level_h, const int64_t *level_w,
                                             const float *locations, const float *weights, void *out, xp_dtype out_type,
                                             void *stream)
{
    using namespace xp;
    if (batch < 0 || Lq < 0 || heads < 0 || d < 0 || levels < 0 || points < 0) return XP_ERR_SHAPE;
    if ((v_type != XP_F32 && v_type != XP_BF16) || (out_type != XP_F32 && out_type != XP_BF16)) return XP_ERR_UNSUPPORTED;
    if (levels > MAX_LEVELS) return XP_ERR_SHAPE;
    const int64_t lim = 0x7fffffffLL;
    if (Lq > lim || heads > lim || d > lim || points > lim || batch > lim) return XP_ERR_SHAPE;
    if (batch == 0 || Lq == 0 || heads == 0 || d == 0) return XP_OK;
    if (levels > 0 && (!level_h || !level_w)) return XP_ERR_NULL;
    DeformParams p{};
    long long S = 0;
    for (int l = 0; l < (int)levels; ++l) {
        if (level_h[l] < 0 || level_w[l] < 0 || level_h[l] > (1 << 24) || level_w[l] > (1 << 24)) return XP_ERR_SHAPE;   // exact in fp32
        p.H[l] = (int)level_h[l];
        p.W[l] = (int)level_w[l];
        p.start[l] = S;
        S += level_h[l] * level_w[l];
        if (S > (1LL << 40)) return XP_ERR_SHAPE;
    }
    const bool samples = levels > 0 && points > 0;
    if (!out || (samples && (!locations || !weights || (S > 0 && !value)))) return XP_ERR_NULL;
    // element counts stay far inside 63 bits: batch*S*heads*d and batch*Lq*heads*levels*points*2
    const long double big = 9.0e18L;
    if ((long double)batch * (long double)S * heads * d > big || (long double)batch * Lq * heads * levels * points * 2 > big ||
        (long double)batch * Lq * heads * d > big)
        return XP_ERR_SHAPE;
    if (samples && ((uintptr_t)locations % 8 || (uintptr_t)weights % 4)) return XP_ERR_ALIGN;

    const bool bf = v_type == XP_BF16, obf = out_type == XP_BF16;
    const int epc = bf ? 8 : 4;
    const bool vec = d % epc == 0 && (uintptr_t)value % 16 == 0 && (uintptr_t)out % 16 == 0;
    if (!vec && ((uintptr_t)value % (bf ? 2 : 4) || (uintptr_t)out % (obf ? 2 : 4))) return XP_ERR_ALIGN;
    p.value = value; p.loc = locations; p.wgt = weights; p.out = out;
    p.S = S; p.Lq = (int)Lq; p.heads = (int)heads; p.d = (int)d; p.levels = (int)levels; p.points = (int)points;
    p.units = (long long)batch * Lq * heads * (vec ? d / epc : d);
    hipStream_t s = (hipStream_t)stream;
    if (vec) {
        LdsPlan plan;
        int lds_bytes = 0;
        dim3 grid;
        if (plan_lds(p, batch, bf ? 2 : 4, epc, plan, lds_bytes, grid)) {
            if (bf) return obf ? launch_lds<true, true>(p, plan, lds_bytes, grid, s) : launch_lds<true, false>(p, plan, lds_bytes, grid, s);
            return obf ? launch_lds<false, true>(p, plan, lds_bytes, grid, s) : launch_lds<false, false>(p, plan, lds_bytes, grid, s);
        }
        if (bf) return obf ? launch<true, true, 8>(p, s) : launch<true, false, 8>(p, s);
        return obf ? launch<false, true, 4>(p, s) : launch<false, false, 4>(p, s);
    }
    if (bf) return obf ? launch<true, true, 1>(p, s) : launch<true, false, 1>(p, s);
    return obf ? launch<false, true, 1>(p, s) : launch<false, false, 1>(p, s);
}
