// Memory-bound operators of the paper's benchmark (Table 5: Activation -- ReLU, Softmax, GeLU,
// Sigmoid; Elementwise -- Add, Sign; Pooling -- Max/Avg/Min/SumPool; LLM -- LayerNorm, RMSNorm;
// Convolution -- Depthwise Conv, which reuses nothing either).
// Each reads its input once and writes its output once: the bound is HBM bandwidth, the matrix
// cores have nothing to do.  Common shape of the kernels: 16-byte loads and stores, fp32
// arithmetic whatever the storage type (fp32 or bf16, output rounded to nearest even), and for the
// row-wise operators the whole row held in registers between the reduction and the write, so that
// it is fetched from memory exactly once.
#include "xp_internal.hpp"

namespace xp {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void lds_void;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }
// two bf16 values, one from each of two words, side by side in one register (the low halves, or the high halves)
__device__ __forceinline__ unsigned pair_lo(unsigned a, unsigned b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ unsigned pair_hi(unsigned a, unsigned b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }
// c + x.lo * w.lo + x.hi * w.hi on bf16 pairs, accumulated in fp32
__device__ __forceinline__ float dot2_bf16(unsigned x, unsigned w, float c)
{
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, x), __builtin_bit_cast(bf2, w), c, false);
}
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));      // round to nearest even
}
__device__ __forceinline__ unsigned short to_bf16(float v) { return (unsigned short)pack_bf16(v, 0.0f); }

// EPC elements per 16-byte input chunk: 4 fp32 or 8 bf16
template <bool BF16> struct Chunk {
    static constexpr int EPC = BF16 ? 8 : 4;
    // STREAM: data that is read exactly once (the operand itself) bypasses the caches' retention;
    // small vectors that every row needs again (gamma, beta) and pooling windows, which overlap, do not
    template <bool STREAM = true>
    __device__ static __forceinline__ void load(const void *p, long long chunk, float (&v)[EPC])
    {
        const u32x4 w = STREAM ? __builtin_nontemporal_load((const u32x4 *)p + chunk) : *((const u32x4 *)p + chunk);
        if constexpr (BF16) {
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[2 * i] = bf16_lo(w[i]); v[2 * i + 1] = bf16_hi(w[i]); }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(w[i]);
        }
    }
};
// store EPC values starting at element e0 of p (aligned to EPC output elements)
template <bool OUT_BF16, int EPC> __device__ __forceinline__ void store_chunk(void *p, long long e0, const float (&v)[EPC])
{
    if constexpr (OUT_BF16) {
        unsigned w[EPC / 2];
#pragma unroll
        for (int i = 0; i < EPC / 2; ++i) w[i] = pack_bf16(v[2 * i], v[2 * i + 1]);
        if constexpr (EPC == 8) __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, (u32x4 *)((unsigned short *)p + e0));
        else __builtin_nontemporal_store(u32x2{w[0], w[1]}, (u32x2 *)((unsigned short *)p + e0));
    } else {
#pragma unroll
        for (int i = 0; i < EPC; i += 4)
            __builtin_nontemporal_store(u32x4{__float_as_uint(v[i]), __float_as_uint(v[i + 1]), __float_as_uint(v[i + 2]),
                                              __float_as_uint(v[i + 3])}, (u32x4 *)((float *)p + e0 + i));
    }
}
template <bool BF16> __device__ __forceinline__ float load1(const void *p, long long i)
{
    if constexpr (BF16) return __uint_as_float((unsigned)((const unsigned short *)p)[i] << 16);
    else return ((const float *)p)[i];
}
template <bool BF16> __device__ __forceinline__ void store1(void *p, long long i, float v)
{
    if constexpr (BF16) ((unsigned short *)p)[i] = to_bf16(v);
    else ((float *)p)[i] = v;
}

// -------------------------------------------------------------------------------- row-wise operators
enum RowOp { SOFTMAX = 0, LAYERNORM = 1, RMSNORM = 2 };

struct RowParams {
    const void *x, *gamma, *beta;
    void *y;
    long long rows, ldx, ldy;
    int cols;
    float eps;
};

// reduction over the TPR threads that share a row (TPR = 64: one wave; else several waves through LDS)
template <int TPR, bool MAX>
__device__ __forceinline__ float row_reduce(float v, float *scratch, int group, int t)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float w = __shfl_xor(v, o);
        v = MAX ? fmaxf(v, w) : v + w;
    }
    if constexpr (TPR > 64) {
        constexpr int NW = TPR / 64;
        __syncthreads();                                   // scratch may still be read from the previous reduction
        if ((t & 63) == 0) scratch[group * NW + (t >> 6)] = v;
        __syncthreads();
        v = scratch[group * NW];
#pragma unroll
        for (int i = 1; i < NW; ++i) v = MAX ? fmaxf(v, scratch[group * NW + i]) : v + scratch[group * NW + i];
    }
    return v;
}

// TPR threads per row, each holding up to NC chunks; the workgroup holds BLOCK / TPR rows.  cols is a
// multiple of EPC, rows start 16-byte aligned, cols / EPC <= TPR * NC.
template <int OP, bool IN_BF16, bool OUT_BF16, int TPR, int NC>
__global__ __launch_bounds__(TPR < 256 ? 256 : TPR) void row_kernel(RowParams p)
{
    constexpr int MAXC = NC;                               // 16-byte chunks of the row that one thread keeps in registers
    constexpr int BLOCK = TPR < 256 ? 256 : TPR, RPB = BLOCK / TPR, EPC = Chunk<IN_BF16>::EPC;
    __shared__ float scratch[BLOCK / 64];
    const int group = threadIdx.x / TPR, t = threadIdx.x % TPR;
    const long long row = (long long)blockIdx.x * RPB + group;
    const bool live = row < p.rows;                        // a dead row group still takes part in the barriers
    const int nchunks = p.cols / EPC;
    const char *xr = (const char *)p.x + (live ? row : 0) * p.ldx * (IN_BF16 ? 2 : 4);

    float v[MAXC][EPC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        // no branch around the load (a chunk past the end reads the row's last chunk and is replaced by the
        // neutral value): at a join the compiler copies the values loaded so far from register to register
        const int ch = t + c * TPR;
        const bool in = live && ch < nchunks;
        Chunk<IN_BF16>::load(xr, min(ch, nchunks - 1), v[c]);
#pragma unroll
        for (int e = 0; e < EPC; ++e) v[c][e] = in ? v[c][e] : (OP == SOFTMAX ? -INFINITY : 0.0f);
    }
    const float inv_n = 1.0f / (float)p.cols;
    float shift = 0.0f, scale = 1.0f;                      // y = (x - shift) * scale [* gamma + beta]
    if constexpr (OP == SOFTMAX) {
        float m = -INFINITY;
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
#pragma unroll
            for (int e = 0; e < EPC; ++e) m = fmaxf(m, v[c][e]);
        m = row_reduce<TPR, true>(m, scratch, group, t);
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                v[c][e] = expf(v[c][e] - m);               // padding lanes hold -inf: exp gives 0
                s += v[c][e];
            }
        s = row_reduce<TPR, false>(s, scratch, group, t);
        scale = 1.0f / s;
    } else if constexpr (OP == LAYERNORM) {
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
#pragma unroll
            for (int e = 0; e < EPC; ++e) s += v[c][e];
        shift = row_reduce<TPR, false>(s, scratch, group, t) * inv_n;
        float q = 0.0f;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const bool in = t + c * TPR < nchunks;         // padding must not count as (0 - mean)^2
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const float d = v[c][e] - shift;
                q += in ? d * d : 0.0f;
            }
        }
        q = row_reduce<TPR, false>(q, scratch, group, t) * inv_n;
        scale = 1.0f / sqrtf(q + p.eps);
    } else {
        float q = 0.0f;
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
#pragma unroll
            for (int e = 0; e < EPC; ++e) q += v[c][e] * v[c][e];
        q = row_reduce<TPR, false>(q, scratch, group, t) * inv_n;
        scale = 1.0f / sqrtf(q + p.eps);
    }
    if (!live) return;
    const float offset = -shift * scale;                   // y = x * scale + offset [* gamma + beta]
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = t + c * TPR;
        if (ch >= nchunks) continue;
        float o[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) o[e] = OP == LAYERNORM ? __builtin_fmaf(v[c][e], scale, offset) : v[c][e] * scale;
        if constexpr (OP != SOFTMAX) {
            if (p.gamma && OP == LAYERNORM && p.beta) {
                float g[EPC], b[EPC];
                Chunk<IN_BF16>::template load<false>(p.gamma, ch, g);
                Chunk<IN_BF16>::template load<false>(p.beta, ch, b);
#pragma unroll
                for (int e = 0; e < EPC; ++e) o[e] = __builtin_fmaf(o[e], g[e], b[e]);
            } else {
                if (p.gamma) {
                    float g[EPC];
                    Chunk<IN_BF16>::template load<false>(p.gamma, ch, g);
#pragma unroll
                    for (int e = 0; e < EPC; ++e) o[e] *= g[e];
                }
                if (OP == LAYERNORM && p.beta) {
                    float b[EPC];
                    Chunk<IN_BF16>::template load<false>(p.beta, ch, b);
#pragma unroll
                    for (int e = 0; e < EPC; ++e) o[e] += b[e];
                }
            }
        }
        store_chunk<OUT_BF16, EPC>(p.y, row * p.ldy + (long long)ch * EPC, o);
    }
}

// any row length and alignment: one workgroup per row, three passes over the row (the second and
// third come from cache for all but very long rows)
template <int OP, bool IN_BF16, bool OUT_BF16>
__global__ __launch_bounds__(256) void row_general_kernel(RowParams p)
{
    __shared__ float scratch[4];
    const int t = threadIdx.x;
    const long long row = blockIdx.x;
    const long long x0 = row * p.ldx, y0 = row * p.ldy;
    const float inv_n = 1.0f / (float)p.cols;
    float shift = 0.0f, scale = 1.0f;
    if constexpr (OP == SOFTMAX) {
        float m = -INFINITY;
        for (int j = t; j < p.cols; j += 256) m = fmaxf(m, load1<IN_BF16>(p.x, x0 + j));
        shift = row_reduce<256, true>(m, scratch, 0, t);
        float s = 0.0f;
        for (int j = t; j < p.cols; j += 256) s += expf(load1<IN_BF16>(p.x, x0 + j) - shift);
        scale = 1.0f / row_reduce<256, false>(s, scratch, 0, t);
        for (int j = t; j < p.cols; j += 256) store1<OUT_BF16>(p.y, y0 + j, expf(load1<IN_BF16>(p.x, x0 + j) - shift) * scale);
        return;
    } else if constexpr (OP == LAYERNORM) {
        float s = 0.0f;
        for (int j = t; j < p.cols; j += 256) s += load1<IN_BF16>(p.x, x0 + j);
        shift = row_reduce<256, false>(s, scratch, 0, t) * inv_n;
        float q = 0.0f;
        for (int j = t; j < p.cols; j += 256) {
            const float d = load1<IN_BF16>(p.x, x0 + j) - shift;
            q += d * d;
        }
        scale = 1.0f / sqrtf(row_reduce<256, false>(q, scratch, 0, t) * inv_n + p.eps);
    } else {
        float q = 0.0f;
        for (int j = t; j < p.cols; j += 256) {
            const float a = load1<IN_BF16>(p.x, x0 + j);
            q += a * a;
        }
        scale = 1.0f / sqrtf(row_reduce<256, false>(q, scratch, 0, t) * inv_n + p.eps);
    }
    for (int j = t; j < p.cols; j += 256) {
        float o = (load1<IN_BF16>(p.x, x0 + j) - shift) * scale;
        if (p.gamma) o *= load1<IN_BF16>(p.gamma, j);
        if (OP == LAYERNORM && p.beta) o += load1<IN_BF16>(p.beta, j);
        store1<OUT_BF16>(p.y, y0 + j, o);
    }
}

bool aligned(const void *p, uintptr_t a) { return ((uintptr_t)p % a) == 0; }

template <int OP, bool IB, bool OB>
hipError_t launch_row(const RowParams &p, hipStream_t stream)
{
    constexpr int EPC = Chunk<IB>::EPC;
    const int isz = IB ? 2 : 4, osz = OB ? 2 : 4;
    const bool vec = p.cols % EPC == 0 && aligned(p.x, 16) && (p.ldx * isz) % 16 == 0 && aligned(p.y, (uintptr_t)EPC * osz) &&
                     p.ldy % EPC == 0 && (!p.gamma || aligned(p.gamma, 16)) && (!p.beta || aligned(p.beta, 16)) &&
                     p.rows <= 0x7fffffffLL;
    const int nchunks = p.cols / EPC;
    const dim3 g1((unsigned)p.rows);
    // Threads per row: a sweep over row lengths (512 .. 32768 columns, fp32 and bf16, all three
    // operators) found two 16-byte chunks per thread the best point -- fewer registers, more waves in
    // flight -- up to 512 threads a row; longer rows take four chunks at 512 threads, then 1024 threads.
    int tpr = 64;
    while (tpr < 512 && (nchunks + tpr - 1) / tpr > 2) tpr *= 2;
    if ((nchunks + tpr - 1) / tpr > 4) tpr = 1024;
    const int need = (nchunks + tpr - 1) / tpr;
    const int nc = need <= 1 ? 1 : (need <= 2 ? 2 : (need <= 4 ? 4 : 8));
    const int block = tpr < 256 ? 256 : tpr;
    const dim3 grid((unsigned)((p.rows + block / tpr - 1) / (block / tpr)));
    bool done = false;
#define XP_ROW(TPR, NC)                                                                                        \
    if (!done && vec && tpr == TPR && nc == NC && need <= 8) {                                                 \
        hipLaunchKernelGGL((row_kernel<OP, IB, OB, TPR, NC>), grid, dim3(block), 0, stream, p);                \
        done = true;                                                                                           \
    }
    // the (threads, chunks) pairs that rule can produce
    XP_ROW(64, 1) XP_ROW(64, 2) XP_ROW(128, 2) XP_ROW(256, 2) XP_ROW(512, 2) XP_ROW(512, 4) XP_ROW(1024, 4) XP_ROW(1024, 8)
#undef XP_ROW
    if (done) return hipGetLastError();
    hipLaunchKernelGGL((row_general_kernel<OP, IB, OB>), g1, dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <int OP>
xp_status row_entry(int64_t rows, int64_t cols, const void *x, xp_dtype x_type, int64_t ldx, const void *gamma,
                    const void *beta, float eps, void *y, xp_dtype y_type, int64_t ldy, void *stream)
{
    if (rows < 0 || cols < 0) return XP_ERR_SHAPE;
    if ((x_type != XP_F32 && x_type != XP_BF16) || (y_type != XP_F32 && y_type != XP_BF16)) return XP_ERR_UNSUPPORTED;
    if (OP != SOFTMAX && (!(eps >= 0.0f) || eps - eps != 0.0f)) return XP_ERR_UNSUPPORTED;     // negative, NaN or infinite
    if (rows == 0 || cols == 0) return XP_OK;
    if (ldx < cols || ldy < cols) return XP_ERR_STRIDE;
    if (!x || !y) return XP_ERR_NULL;
    if (cols > 0x7fffffffLL || rows > 0x7fffffffLL) return XP_ERR_SHAPE;
    const int isz = x_type == XP_BF16 ? 2 : 4, osz = y_type == XP_BF16 ? 2 : 4;
    if (!aligned(x, isz) || !aligned(y, osz) || (gamma && !aligned(gamma, isz)) || (beta && !aligned(beta, isz))) return XP_ERR_ALIGN;
    RowParams p;
    p.x = x; p.gamma = gamma; p.beta = beta; p.y = y;
    p.rows = rows; p.ldx = ldx; p.ldy = ldy; p.cols = (int)cols; p.eps = eps;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (x_type == XP_BF16) e = y_type == XP_BF16 ? launch_row<OP, true, true>(p, s) : launch_row<OP, true, false>(p, s);
    else e = y_type == XP_BF16 ? launch_row<OP, false, true>(p, s) : launch_row<OP, false, false>(p, s);
    return e == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------ element-wise operators
// erfc(z) for z >= 0 as t * exp(-z*z + p(t)), t = 1 / (1 + z/2): p is the degree-8 fit printed by
// fit_erfc.py beside this file (relative error about 1e-6 for z <= 3, 4e-6 for z <= 6, set by the
// fp32 rounding of the exponent).  A dozen instructions where the library erfcf takes several times
// that, which is what makes GELU memory-bound rather than ALU-bound.
__device__ __forceinline__ float erfc_pos(float z)
{
    const float t = __builtin_amdgcn_rcpf(1.0f + 0.5f * z);
    float p = 0.0833144188f;
    p = __builtin_fmaf(p, t, -0.58055824f);
    p = __builtin_fmaf(p, t, 1.53260946f);
    p = __builtin_fmaf(p, t, -1.85293126f);
    p = __builtin_fmaf(p, t, 0.904557347f);
    p = __builtin_fmaf(p, t, -0.259300739f);
    p = __builtin_fmaf(p, t, 0.44532609f);
    p = __builtin_fmaf(p, t, 0.992125869f);
    p = __builtin_fmaf(p, t, -1.26514339f);
    return t * __expf(__builtin_fmaf(-z, z, p));
}

__device__ __forceinline__ float unary_apply(int op, float v)
{
    switch (op) {
    case XP_RELU: return fmaxf(v, 0.0f);
    case XP_GELU: {
        // x * Phi(x), Phi(x) = erfc(-x / sqrt 2) / 2: for x < 0 directly (1 + erf would cancel there),
        // for x >= 0 as 1 - Phi(-x)
        const float h = 0.5f * erfc_pos(fabsf(v) * 0.70710678118654752f);
        return v * (v < 0.0f ? h : 1.0f - h);
    }
    case XP_SIGMOID: return __builtin_amdgcn_rcpf(1.0f + __expf(-v));      // a few ulp; exp overflow gives 1/inf = 0, as it should
    default: return v > 0.0f ? 1.0f : (v < 0.0f ? -1.0f : 0.0f);
    }
}

struct PointParams {
    const void *a, *b;
    void *y;
    long long n;
    int op;                                                 // unary operator, or -1 for a + b
};

template <bool IB, bool OB, bool VEC>
__global__ __launch_bounds__(256) void point_kernel(PointParams p)
{
    constexpr int EPC = Chunk<IB>::EPC;
    const long long tid = (long long)blockIdx.x * 256 + threadIdx.x, nthreads = (long long)gridDim.x * 256;
    if constexpr (VEC) {
        const long long chunks = p.n / EPC;
        for (long long c = tid; c < chunks; c += nthreads) {
            float v[EPC], o[EPC];
            Chunk<IB>::load(p.a, c, v);
            if (p.op < 0) {
                float w[EPC];
                Chunk<IB>::load(p.b, c, w);
#pragma unroll
                for (int e = 0; e < EPC; ++e) o[e] = v[e] + w[e];
            } else {
#pragma unroll
                for (int e = 0; e < EPC; ++e) o[e] = unary_apply(p.op, v[e]);
            }
            store_chunk<OB, EPC>(p.y, c * EPC, o);
        }
        for (long long i = chunks * EPC + tid; i < p.n; i += nthreads) {
            const float v = load1<IB>(p.a, i);
            store1<OB>(p.y, i, p.op < 0 ? v + load1<IB>(p.b, i) : unary_apply(p.op, v));
        }
    } else {
        for (long long i = tid; i < p.n; i += nthreads) {
            const float v = load1<IB>(p.a, i);
            store1<OB>(p.y, i, p.op < 0 ? v + load1<IB>(p.b, i) : unary_apply(p.op, v));
        }
    }
}

xp_status point_entry(int op, int64_t n, const void *a, const void *b, xp_dtype x_type, void *y, xp_dtype y_type, void *stream)
{
    if (n < 0) return XP_ERR_SHAPE;
    if ((x_type != XP_F32 && x_type != XP_BF16) || (y_type != XP_F32 && y_type != XP_BF16)) return XP_ERR_UNSUPPORTED;
    if (op > XP_SIGN) return XP_ERR_UNSUPPORTED;
    if (n == 0) return XP_OK;
    if (!a || !y || (op < 0 && !b)) return XP_ERR_NULL;
    const int isz = x_type == XP_BF16 ? 2 : 4, osz = y_type == XP_BF16 ? 2 : 4;
    if (!aligned(a, isz) || !aligned(y, osz) || (op < 0 && !aligned(b, isz))) return XP_ERR_ALIGN;
    PointParams p;
    p.a = a; p.b = b; p.y = y; p.n = n; p.op = op;
    const int epc = x_type == XP_BF16 ? 8 : 4;
    const bool vec = aligned(a, 16) && (op >= 0 || aligned(b, 16)) && aligned(y, (uintptr_t)epc * osz);
    const long long work = vec ? (n + epc - 1) / epc : n;
    long long blocks = (work + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;               // grid-stride beyond 32 workgroups per compute unit
    const dim3 grid((unsigned)blocks), block(256);
    hipStream_t s = (hipStream_t)stream;
#define XP_POINT(IB, OB)                                                                              \
    do {                                                                                              \
        if (vec) hipLaunchKernelGGL((point_kernel<IB, OB, true>), grid, block, 0, s, p);              \
        else hipLaunchKernelGGL((point_kernel<IB, OB, false>), grid, block, 0, s, p);                 \
    } while (0)
    if (x_type == XP_BF16) { if (y_type == XP_BF16) XP_POINT(true, true); else XP_POINT(true, false); }
    else { if (y_type == XP_BF16) XP_POINT(false, true); else XP_POINT(false, false); }
#undef XP_POINT
    return hipGetLastError() == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------------- pooling
struct PoolParams {
    const void *x;
    void *y;
    int op;
    long long total;                                        // work items: output pixels x channel chunks (or channels)
    int H, W, C, R, S, P, Q, sh, sw, ph, pw;
};

// one work item = one output pixel and EPC consecutive channels (VEC) or one channel.  WIN > 0: the
// window is WIN x WIN, known at compile time, so that its loads are all issued before the first is used.
// OP >= 0: the reduction is known at compile time too (the windowed kernels): no selects per element, and an
// output whose window lies inside the image combines its WIN x WIN values without any test.  The kernel is bound
// by vector instructions, not by memory, when it tests every element for the operation and for being inside.
template <bool IB, bool OB, bool VEC, int WIN, int OP = -1>
__global__ __launch_bounds__(256) void pool_kernel(PoolParams p)
{
    constexpr int EPC = VEC ? Chunk<IB>::EPC : 1;
    const int cc = p.C / EPC;                               // channel groups per pixel
    // neighbouring outputs share input rows: XCD-contiguous numbering (grid is a multiple of 8)
    for (long long w = (long long)xcd_chunked(blockIdx.x, gridDim.x) * 256 + threadIdx.x; w < p.total; w += (long long)gridDim.x * 256) {
        const int cg = (int)(w % cc);
        long long pix = w / cc;
        const int q = (int)(pix % p.Q);
        pix /= p.Q;
        const int op_ = (int)(pix % p.P);
        const long long n = pix / p.P;
        float acc[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] = 0.0f;
        int inside = 0;
        auto take = [&](const float (&v)[EPC]) {
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const int op = OP >= 0 ? OP : p.op;
                if (inside == 0) acc[e] = v[e];
                else if (op == XP_POOL_MAX) acc[e] = fmaxf(acc[e], v[e]);
                else if (op == XP_POOL_MIN) acc[e] = fminf(acc[e], v[e]);
                else acc[e] += v[e];
            }
            ++inside;
        };
        auto fetch = [&](int h, int x, float (&v)[EPC]) {
            const long long pixel = (n * p.H + h) * p.W + x;
            if constexpr (VEC) Chunk<IB>::template load<false>(p.x, pixel * cc + cg, v);
            else v[0] = load1<IB>(p.x, pixel * p.C + cg);
        };
        if constexpr (WIN > 0) {
            float v[WIN * WIN][EPC];
            bool in[WIN * WIN];
#pragma unroll
            for (int r = 0; r < WIN; ++r)
#pragma unroll
                for (int s = 0; s < WIN; ++s) {
                    const int h = op_ * p.sh + r - p.ph, x = q * p.sw + s - p.pw;
                    in[r * WIN + s] = h >= 0 && h < p.H && x >= 0 && x < p.W;
                    // positions outside the image load the nearest pixel inside (never used): no branch around a load
                    fetch(min(max(h, 0), p.H - 1), min(max(x, 0), p.W - 1), v[r * WIN + s]);
                }
            bool all_in = true;
#pragma unroll
            for (int i = 0; i < WIN * WIN; ++i) all_in = all_in && in[i];
            if (OP >= 0 && all_in) {
                // the window lies inside the image (all but the border outputs)
#pragma unroll
                for (int e = 0; e < EPC; ++e) {
                    float a = v[0][e];
#pragma unroll
                    for (int i = 1; i < WIN * WIN; ++i) {
                        if (OP == XP_POOL_MAX) a = fmaxf(a, v[i][e]);
                        else if (OP == XP_POOL_MIN) a = fminf(a, v[i][e]);
                        else a += v[i][e];
                    }
                    acc[e] = a;
                }
                inside = WIN * WIN;
            } else {
#pragma unroll
                for (int i = 0; i < WIN * WIN; ++i)
                    if (in[i]) take(v[i]);
            }
        } else {
            for (int r = 0; r < p.R; ++r) {
                const int h = op_ * p.sh + r - p.ph;
                if (h < 0 || h >= p.H) continue;
                for (int s = 0; s < p.S; ++s) {
                    const int x = q * p.sw + s - p.pw;
                    if (x < 0 || x >= p.W) continue;
                    float v[EPC];
                    fetch(h, x, v);
                    take(v);
                }
            }
        }
        if ((OP >= 0 ? OP : p.op) == XP_POOL_AVG && inside > 0) {
            const float inv = 1.0f / (float)inside;
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[e] *= inv;
        }
        if constexpr (VEC) store_chunk<OB, EPC>(p.y, w * EPC, acc);
        else store1<OB>(p.y, w, acc[0]);
    }
}

// ------------------------------------------------------------------------------- depthwise convolution
// Same work decomposition as pooling (one output pixel x EPC channels per work item), with a weight
// per (tap, channel).  WIN > 0: a WIN x WIN window with channel-minor weights, loads issued up front.
struct DwParams {
    const void *x, *w;
    void *y;
    long long total;
    long long tiles;                                        // workgroups with work in the tiled kernel
    int H, W, C, R, S, P, Q, sh, sw, ph, pw;
    int channel_minor;                                      // w(c,r,s) at (r*S + s)*C + c, else (c*R + r)*S + s
};

template <bool IB, bool OB, bool VEC, int WIN>
__global__ __launch_bounds__(256) void depthwise_kernel(DwParams p)
{
    constexpr int EPC = VEC ? Chunk<IB>::EPC : 1;
    const int cc = p.C / EPC;
    for (long long wi = (long long)xcd_chunked(blockIdx.x, gridDim.x) * 256 + threadIdx.x; wi < p.total; wi += (long long)gridDim.x * 256) {
        const int cg = (int)(wi % cc);
        long long pix = wi / cc;
        const int q = (int)(pix % p.Q);
        pix /= p.Q;
        const int op_ = (int)(pix % p.P);
        const long long n = pix / p.P;
        float acc[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] = 0.0f;
        auto fetch = [&](int h, int x, float (&v)[EPC]) {
            const long long pixel = (n * p.H + h) * p.W + x;
            if constexpr (VEC) Chunk<IB>::template load<false>(p.x, pixel * cc + cg, v);
            else v[0] = load1<IB>(p.x, pixel * p.C + cg);
        };
        auto weights = [&](int r, int s, float (&g)[EPC]) {
            if (p.channel_minor) {
                if constexpr (VEC) Chunk<IB>::template load<false>(p.w, (long long)(r * p.S + s) * cc + cg, g);
                else g[0] = load1<IB>(p.w, (long long)(r * p.S + s) * p.C + cg);
            } else {
#pragma unroll
                for (int e = 0; e < EPC; ++e) g[e] = load1<IB>(p.w, ((long long)(cg * EPC + e) * p.R + r) * p.S + s);
            }
        };
        if constexpr (WIN > 0) {
            float v[WIN * WIN][EPC], g[WIN * WIN][EPC];
            bool in[WIN * WIN];
#pragma unroll
            for (int r = 0; r < WIN; ++r)
#pragma unroll
                for (int s = 0; s < WIN; ++s) {
                    const int h = op_ * p.sh + r - p.ph, x = q * p.sw + s - p.pw;
                    in[r * WIN + s] = h >= 0 && h < p.H && x >= 0 && x < p.W;
                    fetch(min(max(h, 0), p.H - 1), min(max(x, 0), p.W - 1), v[r * WIN + s]);   // clamped: no branch around a load
                    Chunk<IB>::template load<false>(p.w, (long long)(r * WIN + s) * cc + cg, g[r * WIN + s]);
                }
#pragma unroll
            for (int i = 0; i < WIN * WIN; ++i)
#pragma unroll
                for (int e = 0; e < EPC; ++e) acc[e] = __builtin_fmaf(in[i] ? v[i][e] : 0.0f, g[i][e], acc[e]);
        } else {
            for (int r = 0; r < p.R; ++r) {
                const int h = op_ * p.sh + r - p.ph;
                if (h < 0 || h >= p.H) continue;
                for (int s = 0; s < p.S; ++s) {
                    const int x = q * p.sw + s - p.pw;
                    if (x < 0 || x >= p.W) continue;
                    float v[EPC], g[EPC];
                    fetch(h, x, v);
                    weights(r, s, g);
#pragma unroll
                    for (int e = 0; e < EPC; ++e) acc[e] = __builtin_fmaf(v[e], g[e], acc[e]);
                }
            }
        }
        if constexpr (VEC) store_chunk<OB, EPC>(p.y, wi * EPC, acc);
        else store1<OB>(p.y, wi, acc[0]);
    }
}

// 3 x 3, stride 1, channel-minor weights, whole 16-byte channel chunks: the common depthwise case.
// The one-work-item-per-output kernel above issues 18 loads per output chunk (9 pixels, 9 weights)
// and is bound by the rate of L1 requests, not by HBM.  Here a workgroup stages the input patch of
// an 8 x 16 tile of outputs for 8 channel chunks (10 x 18 pixels, 1.4 loads per output chunk, all
// issued up front, written to LDS by the loads themselves) in LDS, keeps its 9 weight chunks in registers,
// and reads the taps from LDS.
constexpr int DW_TH = 8, DW_TW = 16, DW_CG = 8;            // output rows, columns and channel chunks per workgroup
constexpr int DW_PH = DW_TH + 2, DW_PW = DW_TW + 2;

template <bool IB, bool OB>
__global__ __launch_bounds__(256) void depthwise3x3_tile_kernel(DwParams p)
{
    constexpr int EPC = Chunk<IB>::EPC;
    __shared__ u32x4 patch[(DW_PH * DW_PW * DW_CG + 255) / 256 * 256];   // [patch row][patch column][channel chunk], padded to whole rounds of loads
    const int cc = p.C / EPC;
    const int t = threadIdx.x;
    const int tiles_w = (p.Q + DW_TW - 1) / DW_TW, tiles_h = (p.P + DW_TH - 1) / DW_TH, cblocks = (cc + DW_CG - 1) / DW_CG;
    // neighbouring tiles share their border rows and columns: XCD-contiguous numbering (grid is a multiple of 8)
    long long b = xcd_chunked(blockIdx.x, gridDim.x);
    if (b >= (long long)p.tiles) return;
    const int cb = b % cblocks; b /= cblocks;
    const int tw = b % tiles_w; b /= tiles_w;
    const int th = b % tiles_h;
    const long long n = b / tiles_h;
    const int p0 = th * DW_TH, q0 = tw * DW_TW, cg0 = cb * DW_CG;

    // stage the patch: rows p0 - ph .. +DW_PH, columns q0 - pw .. +DW_PW; zeros outside the image or past the last chunk.
    constexpr int PATCH = DW_PH * DW_PW * DW_CG, ROUNDS = (PATCH + 255) / 256;
    // The loads write LDS directly, 16 bytes per lane at consecutive addresses: lane i of the workgroup's round
    // `it` fills chunk it * 256 + i of the patch, which is the patch's own order.  A position outside the image,
    // past the last channel chunk or past the patch gets a byte offset beyond the range of the image's buffer
    // descriptor, for which the load writes zeros (the patch array is padded to whole rounds for the latter).
    const __amdgpu_buffer_rsrc_t image = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u32x4 *>((const u32x4 *)p.x + n * p.H * p.W * cc), 0, (unsigned)(p.H * p.W * cc) * 16u, 0x00020000);
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
#pragma unroll
    for (int it = 0; it < ROUNDS; ++it) {                  // all loads are in flight together
        const int i = t + it * 256;
        const int pc = i % DW_CG, col = (i / DW_CG) % DW_PW, row = i / (DW_CG * DW_PW);
        const int h = p0 - p.ph + row, x = q0 - p.pw + col;
        const bool valid = (h >= 0) & (h < p.H) & (x >= 0) & (x < p.W) & (cg0 + pc < cc) & (i < PATCH);
        const unsigned off = valid ? ((unsigned)(h * p.W + x) * (unsigned)cc + (unsigned)(cg0 + pc)) * 16u : 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(image, (lds_void *)(patch + it * 256 + wave * 64), 16, off, 0, 0, 0);
    }
    // this thread's channel chunk and its 9 weight chunks (a chunk past the last one computes with the last
    // one's weights and is not stored)
    const int cg = t % DW_CG;
    const bool live_c = cg0 + cg < cc;
    if constexpr (IB) {
        // bf16: taps in pairs through the two-element dot product (one instruction for two taps of a channel,
        // fp32 accumulation).  Channels are the minor index in memory, so a pair's two taps are brought into one
        // register by a byte permute: (rows 0, 1) of each tap column, (columns 0, 1) of row 2; tap (2, 2) stays a
        // plain multiply-add.  Per pair of neighbouring outputs: 48 permutes + 64 dot products + 16 widenings +
        // 16 multiply-adds, against 96 widenings + 144 multiply-adds one tap at a time (the kernel is bound by
        // its vector instructions), and 40 weight registers instead of 72.
        u32x4 wr[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) wr[k] = *((const u32x4 *)p.w + (long long)k * cc + min(cg0 + cg, cc - 1));
        unsigned wv[3][EPC], wh[EPC];
        float ws[EPC];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                wv[k][2 * i] = pair_lo(wr[k][i], wr[3 + k][i]);
                wv[k][2 * i + 1] = pair_hi(wr[k][i], wr[3 + k][i]);
            }
            wh[2 * i] = pair_lo(wr[6][i], wr[7][i]);
            wh[2 * i + 1] = pair_hi(wr[6][i], wr[7][i]);
            ws[2 * i] = bf16_lo(wr[8][i]);
            ws[2 * i + 1] = bf16_hi(wr[8][i]);
        }
        __builtin_amdgcn_s_waitcnt(0x0070);              // the patch has arrived in LDS (vmcnt 0, lgkmcnt 0)
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int grp = t / DW_CG + j * (256 / DW_CG), r = grp / (DW_TW / 2), c0 = (grp % (DW_TW / 2)) * 2;
            float acc[2][EPC];
#pragma unroll
            for (int o = 0; o < 2; ++o)
#pragma unroll
                for (int e = 0; e < EPC; ++e) acc[o][e] = 0.0f;
#pragma unroll
            for (int dc = 0; dc < 4; ++dc) {               // rows 0 and 1 of the four input columns under the pair
                const u32x4 v0 = patch[(r * DW_PW + c0 + dc) * DW_CG + cg];
                const u32x4 v1 = patch[((r + 1) * DW_PW + c0 + dc) * DW_CG + cg];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const unsigned lo = pair_lo(v0[i], v1[i]), hi = pair_hi(v0[i], v1[i]);
#pragma unroll
                    for (int o = 0; o < 2; ++o) {
                        const int k = dc - o;               // tap column of this input for output o
                        if (k >= 0 && k < 3) {
                            acc[o][2 * i] = dot2_bf16(lo, wv[k][2 * i], acc[o][2 * i]);
                            acc[o][2 * i + 1] = dot2_bf16(hi, wv[k][2 * i + 1], acc[o][2 * i + 1]);
                        }
                    }
                }
            }
            u32x4 v2[4];                                    // row 2
#pragma unroll
            for (int dc = 0; dc < 4; ++dc) v2[dc] = patch[((r + 2) * DW_PW + c0 + dc) * DW_CG + cg];
#pragma unroll
            for (int o = 0; o < 2; ++o)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[o][2 * i] = dot2_bf16(pair_lo(v2[o][i], v2[o + 1][i]), wh[2 * i], acc[o][2 * i]);
                    acc[o][2 * i + 1] = dot2_bf16(pair_hi(v2[o][i], v2[o + 1][i]), wh[2 * i + 1], acc[o][2 * i + 1]);
                    acc[o][2 * i] = __builtin_fmaf(bf16_lo(v2[o + 2][i]), ws[2 * i], acc[o][2 * i]);
                    acc[o][2 * i + 1] = __builtin_fmaf(bf16_hi(v2[o + 2][i]), ws[2 * i + 1], acc[o][2 * i + 1]);
                }
            const int op_ = p0 + r;
#pragma unroll
            for (int o = 0; o < 2; ++o) {
                const int oq = q0 + c0 + o;
                if (op_ < p.P && oq < p.Q && live_c)
                    store_chunk<OB, EPC>(p.y, (((n * p.P + op_) * p.Q + oq) * cc + cg0 + cg) * EPC, acc[o]);
            }
        }
        return;
    }
    float w[9][EPC];
#pragma unroll
    for (int k = 0; k < 9; ++k) Chunk<IB>::template load<false>(p.w, (long long)k * cc + min(cg0 + cg, cc - 1), w[k]);
    __builtin_amdgcn_s_waitcnt(0x0070);              // the patch has arrived in LDS (vmcnt 0, lgkmcnt 0)
    __syncthreads();
    // 128 output pixels x 8 chunks over 256 threads: 4 pixels per thread, as two pairs of neighbours in a row, so
    // that the 3 x 4 input chunks under a pair are read from LDS and widened to fp32 once (12 instead of 18
    // reads; the kernel is bound by its vector instructions, a third of which were these conversions).  Four in a
    // row would share more, but the registers of four accumulator sets cost a wave of occupancy (28.2 against 27.2 us).
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int grp = t / DW_CG + j * (256 / DW_CG), r = grp / (DW_TW / 2), c0 = (grp % (DW_TW / 2)) * 2;
        float acc[2][EPC];
#pragma unroll
        for (int o = 0; o < 2; ++o)
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[o][e] = 0.0f;
#pragma unroll
        for (int dr = 0; dr < 3; ++dr)
#pragma unroll
            for (int dc = 0; dc < 4; ++dc) {
                const u32x4 v = patch[((r + dr) * DW_PW + c0 + dc) * DW_CG + cg];
                float x[EPC];
                if constexpr (IB) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_lo(v[i]); x[2 * i + 1] = bf16_hi(v[i]); }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(v[i]);
                }
#pragma unroll
                for (int o = 0; o < 2; ++o) {
                    const int k = dc - o;                   // tap column of this input for output o
                    if (k >= 0 && k < 3) {
#pragma unroll
                        for (int e = 0; e < EPC; ++e) acc[o][e] = __builtin_fmaf(x[e], w[dr * 3 + k][e], acc[o][e]);
                    }
                }
            }
        const int op_ = p0 + r;
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            const int oq = q0 + c0 + o;
            if (op_ < p.P && oq < p.Q && live_c)
                store_chunk<OB, EPC>(p.y, (((n * p.P + op_) * p.Q + oq) * cc + cg0 + cg) * EPC, acc[o]);
        }
    }
}

}  // namespace
}  // namespace xp

using namespace xp;

extern "C" {

xp_status xp_softmax(int64_t rows, int64_t cols, const void *x, xp_dtype x_type, int64_t ldx,
                     void *y, xp_dtype y_type, int64_t ldy, void *stream)
{
    return row_entry<SOFTMAX>(rows, cols, x, x_type, ldx, nullptr, nullptr, 0.0f, y, y_type, ldy, stream);
}

xp_status xp_layernorm(int64_t rows, int64_t cols, const void *x, xp_dtype x_type, int64_t ldx,
                       const void *gamma, const void *beta, float eps, void *y, xp_dtype y_type, int64_t ldy, void *stream)
{
    return row_entry<LAYERNORM>(rows, cols, x, x_type, ldx, gamma, beta, eps, y, y_type, ldy, stream);
}

xp_status xp_rmsnorm(int64_t rows, int64_t cols, const void *x, xp_dtype x_type, int64_t ldx,
                     const void *gamma, float eps, void *y, xp_dtype y_type, int64_t ldy, void *stream)
{
    return row_entry<RMSNORM>(rows, cols, x, x_type, ldx, gamma, nullptr, eps, y, y_type, ldy, stream);
}

xp_status xp_unary(xp_unary_op op, int64_t n, const void *x, xp_dtype x_type, void *y, xp_dtype y_type, void *stream)
{
    if (op < XP_RELU || op > XP_SIGN) return XP_ERR_UNSUPPORTED;
    return point_entry((int)op, n, x, nullptr, x_type, y, y_type, stream);
}

xp_status xp_add(int64_t n, const void *a, const void *b, xp_dtype type, void *y, xp_dtype y_type, void *stream)
{
    return point_entry(-1, n, a, b, type, y, y_type, stream);
}

xp_status xp_pool2d_nhwc(xp_pool_op op, int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                         int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                         const void *x, xp_dtype x_type, void *y, xp_dtype y_type, void *stream)
{
    if (N < 0 || H < 0 || W < 0 || C < 0) return XP_ERR_SHAPE;
    if (R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return XP_ERR_SHAPE;
    if (op < XP_POOL_MAX || op > XP_POOL_SUM) return XP_ERR_UNSUPPORTED;
    if ((x_type != XP_F32 && x_type != XP_BF16) || (y_type != XP_F32 && y_type != XP_BF16)) return XP_ERR_UNSUPPORTED;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return XP_OK;                // empty output
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N == 0 || C == 0) return XP_OK;
    if (!x || !y) return XP_ERR_NULL;
    const int isz = x_type == XP_BF16 ? 2 : 4, osz = y_type == XP_BF16 ? 2 : 4;
    if (!aligned(x, isz) || !aligned(y, osz)) return XP_ERR_ALIGN;
    const int64_t lim = 0x7fffffffLL;
    if (H > lim || W > lim || C > lim || R > lim || S > lim || stride_h > lim || stride_w > lim || pad_h > lim || pad_w > lim)
        return XP_ERR_SHAPE;
    const int epc = x_type == XP_BF16 ? 8 : 4;
    const bool vec = C % epc == 0 && aligned(x, 16) && aligned(y, (uintptr_t)epc * osz);
    PoolParams p;
    p.x = x; p.y = y; p.op = (int)op;
    p.total = N * P * Q * (vec ? C / epc : C);
    p.H = (int)H; p.W = (int)W; p.C = (int)C; p.R = (int)R; p.S = (int)S; p.P = (int)P; p.Q = (int)Q;
    p.sh = (int)stride_h; p.sw = (int)stride_w; p.ph = (int)pad_h; p.pw = (int)pad_w;
    long long blocks = (p.total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    blocks = (blocks + 7) / 8 * 8;                          // see xcd_chunked
    const dim3 grid((unsigned)blocks), block(256);
    hipStream_t s = (hipStream_t)stream;
    const int win = (R == S && (R == 2 || R == 3) && vec) ? (int)R : 0;
#define XP_POOL(IB, OB)                                                                             \
    do {                                                                                            \
        if (win == 3 && p.op == XP_POOL_MAX) hipLaunchKernelGGL((pool_kernel<IB, OB, true, 3, XP_POOL_MAX>), grid, block, 0, s, p); \
        else if (win == 3 && p.op == XP_POOL_AVG) hipLaunchKernelGGL((pool_kernel<IB, OB, true, 3, XP_POOL_AVG>), grid, block, 0, s, p); \
        else if (win == 2 && p.op == XP_POOL_MAX) hipLaunchKernelGGL((pool_kernel<IB, OB, true, 2, XP_POOL_MAX>), grid, block, 0, s, p); \
        else if (win == 2 && p.op == XP_POOL_AVG) hipLaunchKernelGGL((pool_kernel<IB, OB, true, 2, XP_POOL_AVG>), grid, block, 0, s, p); \
        else if (win == 3) hipLaunchKernelGGL((pool_kernel<IB, OB, true, 3>), grid, block, 0, s, p);     \
        else if (win == 2) hipLaunchKernelGGL((pool_kernel<IB, OB, true, 2>), grid, block, 0, s, p); \
        else if (vec) hipLaunchKernelGGL((pool_kernel<IB, OB, true, 0>), grid, block, 0, s, p);     \
        else hipLaunchKernelGGL((pool_kernel<IB, OB, false, 0>), grid, block, 0, s, p);             \
    } while (0)
    if (x_type == XP_BF16) { if (y_type == XP_BF16) XP_POOL(true, true); else XP_POOL(true, false); }
    else { if (y_type == XP_BF16) XP_POOL(false, true); else XP_POOL(false, false); }
#undef XP_POOL
    return hipGetLastError() == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

xp_status xp_depthwise_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                                   int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                   const void *x, xp_dtype x_type, const void *w, xp_dtype w_type, xp_filter_layout w_layout,
                                   void *y, xp_dtype y_type, void *stream)
{
    if (N < 0 || H < 0 || W < 0 || C < 0) return XP_ERR_SHAPE;
    if (R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return XP_ERR_SHAPE;
    if (w_layout != XP_FILTER_KRSC && w_layout != XP_FILTER_RSCK) return XP_ERR_UNSUPPORTED;
    if ((x_type != XP_F32 && x_type != XP_BF16) || w_type != x_type || (y_type != XP_F32 && y_type != XP_BF16)) return XP_ERR_UNSUPPORTED;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return XP_OK;                // empty output
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N == 0 || C == 0) return XP_OK;
    if (!x || !w || !y) return XP_ERR_NULL;
    const int isz = x_type == XP_BF16 ? 2 : 4, osz = y_type == XP_BF16 ? 2 : 4;
    if (!aligned(x, isz) || !aligned(w, isz) || !aligned(y, osz)) return XP_ERR_ALIGN;
    const int64_t lim = 0x7fffffffLL;
    if (H > lim || W > lim || C > lim || R > lim || S > lim || stride_h > lim || stride_w > lim || pad_h > lim || pad_w > lim ||
        R * S > lim)
        return XP_ERR_SHAPE;
    const int epc = x_type == XP_BF16 ? 8 : 4;
    const bool minor = w_layout == XP_FILTER_RSCK;
    const bool vec = C % epc == 0 && aligned(x, 16) && aligned(y, (uintptr_t)epc * osz) && (!minor || aligned(w, 16));
    DwParams p;
    p.x = x; p.w = w; p.y = y;
    p.total = N * P * Q * (vec ? C / epc : C);
    p.H = (int)H; p.W = (int)W; p.C = (int)C; p.R = (int)R; p.S = (int)S; p.P = (int)P; p.Q = (int)Q;
    p.sh = (int)stride_h; p.sw = (int)stride_w; p.ph = (int)pad_h; p.pw = (int)pad_w;
    p.channel_minor = minor ? 1 : 0;
    long long blocks = (p.total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    blocks = (blocks + 7) / 8 * 8;
    const dim3 grid((unsigned)blocks), block(256);
    hipStream_t s = (hipStream_t)stream;
    const bool win3 = vec && minor && R == 3 && S == 3;
    // stride 1 and an image of several tiles: the LDS-tiled kernel
    const bool tiled = win3 && stride_h == 1 && stride_w == 1 && P >= DW_TH && Q >= DW_TW && H * W * (C / epc) * 16 <= lim;
    const long long tiles = N * ((P + DW_TH - 1) / DW_TH) * ((Q + DW_TW - 1) / DW_TW) * ((C / epc + DW_CG - 1) / DW_CG);
    p.tiles = tiles;
#define XP_DW(IB, OB)                                                                                  \
    do {                                                                                               \
        if (tiled && tiles <= 0x7ffffff0LL)                                                            \
            hipLaunchKernelGGL((depthwise3x3_tile_kernel<IB, OB>), dim3((unsigned)((tiles + 7) / 8 * 8)), block, 0, s, p); \
        else if (win3) hipLaunchKernelGGL((depthwise_kernel<IB, OB, true, 3>), grid, block, 0, s, p);  \
        else if (vec) hipLaunchKernelGGL((depthwise_kernel<IB, OB, true, 0>), grid, block, 0, s, p);   \
        else hipLaunchKernelGGL((depthwise_kernel<IB, OB, false, 0>), grid, block, 0, s, p);           \
    } while (0)
    if (x_type == XP_BF16) { if (y_type == XP_BF16) XP_DW(true, true); else XP_DW(true, false); }
    else { if (y_type == XP_BF16) XP_DW(false, true); else XP_DW(false, false); }
#undef XP_DW
    return hipGetLastError() == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

}  // extern "C"
