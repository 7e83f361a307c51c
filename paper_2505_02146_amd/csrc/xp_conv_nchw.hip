// Conv2D NCHW (Table 5 of the paper) by a change of layout: the activations are transposed to NHWC and
// the KCRS filter to KRSC in a caller-provided workspace (LDS-tiled passes, both sides coalesced), the
// NHWC implicit-GEMM kernels do the work, and their epilogue writes the result straight into the
// N x Cout x P x Q planes (Problem::c_plane).  The MFMA kernels want the reduction index (channels)
// contiguous, which is what NHWC is; the output has no such constraint.
#include "xp_internal.hpp"

#include <atomic>

namespace xp {
namespace {

constexpr int TT = 64;                                   // transpose tile edge

struct TrParams {
    const void *in;
    void *out;
    long long rows, cols;                                // of one input matrix; the output is cols x rows
};

// out[b][c][r] = in[b][r][c]; one 64 x 64 tile per workgroup, through LDS so that both the reads
// (along c) and the writes (along r) are contiguous
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(TrParams p)
{
    __shared__ T tile[TT][TT + 1];
    const long long b = blockIdx.z;
    const long long r0 = (long long)blockIdx.y * TT, c0 = (long long)blockIdx.x * TT;
    const T *in = (const T *)p.in + b * p.rows * p.cols;
    T *out = (T *)p.out + b * p.rows * p.cols;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < TT; i += 4) {
        const long long r = r0 + ty + i, c = c0 + tx;
        if (r < p.rows && c < p.cols) tile[ty + i][tx] = in[r * p.cols + c];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TT; i += 4) {
        const long long c = c0 + ty + i, r = r0 + tx;
        if (c < p.cols && r < p.rows) out[c * p.rows + r] = tile[tx][ty + i];
    }
}

// 2-byte elements, rows and cols multiples of 8, both buffers 16-byte aligned: 16-byte global accesses
// on both sides.  Reading, a lane takes 8 consecutive columns of a row (8 lanes a row of the tile);
// writing, 8 consecutive rows of a column gathered from LDS (8 lanes a 128-byte output segment).
// The LDS pitch of 33 words puts the 8 rows of a lane's gather in 8 different banks.
__global__ __launch_bounds__(256) void transpose16_kernel(TrParams p)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    constexpr int PITCH = TT + 2;                         // elements: 33 words
    __shared__ __attribute__((aligned(16))) unsigned short tile[TT * PITCH];
    const long long b = blockIdx.z;
    const long long r0 = (long long)blockIdx.y * TT, c0 = (long long)blockIdx.x * TT;
    const unsigned short *in = (const unsigned short *)p.in + b * p.rows * p.cols;
    unsigned short *out = (unsigned short *)p.out + b * p.rows * p.cols;
    const int t = threadIdx.x, chunk = t & 7, line = t >> 3;      // 8 chunks of 8 elements, 32 lines per pass
    u32x4 v[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const long long r = r0 + line + 32 * i, c = c0 + chunk * 8;
        v[i] = u32x4{0u, 0u, 0u, 0u};
        if (r < p.rows && c < p.cols) v[i] = __builtin_nontemporal_load((const u32x4 *)(in + r * p.cols + c));
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        unsigned *dst = (unsigned *)(tile + (line + 32 * i) * PITCH + chunk * 8);
#pragma unroll
        for (int k = 0; k < 4; ++k) dst[k] = v[i][k];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int cl = line + 32 * i;                     // column of the tile = output row
        const long long c = c0 + cl, r = r0 + chunk * 8;
        if (c < p.cols && r < p.rows) {
            unsigned w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                w[k] = (unsigned)tile[(chunk * 8 + 2 * k) * PITCH + cl] | ((unsigned)tile[(chunk * 8 + 2 * k + 1) * PITCH + cl] << 16);
            __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, (u32x4 *)(out + c * p.rows + r));
        }
    }
}

hipError_t transpose(const void *in, void *out, int64_t batch, int64_t rows, int64_t cols, int esz, hipStream_t s)
{
    TrParams p;
    p.in = in; p.out = out; p.rows = rows; p.cols = cols;
    const dim3 grid((unsigned)((cols + TT - 1) / TT), (unsigned)((rows + TT - 1) / TT), (unsigned)batch);
    if (esz == 2 && rows % 8 == 0 && cols % 8 == 0 && (uintptr_t)in % 16 == 0 && (uintptr_t)out % 16 == 0)
        hipLaunchKernelGGL(transpose16_kernel, grid, dim3(256), 0, s, p);
    else if (esz == 2) hipLaunchKernelGGL(transpose_kernel<unsigned short>, grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL(transpose_kernel<unsigned int>, grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

size_t round256(size_t x) { return (x + 255) / 256 * 256; }


// The library's own layout-change buffer, for callers that cannot hand over a workspace they allocated
// (xp_conv2d_nchw_static).  One copy per GPU, held from the moment the library is loaded there until the
// process ends.  In host code the array's name is only a handle: its device address is looked up once per
// device (static_scratch) and that pointer is what kernels and size checks get.
constexpr size_t STATIC_BYTES = (size_t)64 << 20;
__device__ __align__(256) unsigned char scratch[STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
std::atomic<void *> scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device (looked up on the first call there; no allocation).
xp_status static_scratch(void **out)
{
    int d = -1;
    if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= MAX_DEVICES) return XP_ERR_LAUNCH;
    void *p = scratch_ptr[d].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return XP_ERR_LAUNCH;
        scratch_ptr[d].store(p, std::memory_order_release);      // every thread finds the same address: a race here is benign
    }
    *out = p;
    return XP_OK;
}

xp_status conv2d_nchw_in(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                         int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                         const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                         void *output, xp_dtype out_type, void *workspace, size_t workspace_bytes, bool is_static, void *stream)
{
    // the NHWC entry's own validation, on the pointers it will actually see (checked before anything is launched)
    if (N < 0 || H < 0 || W < 0 || Cin < 0 || Cout < 0) return XP_ERR_SHAPE;
    if (R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return XP_ERR_SHAPE;
    if (in_type != w_type || (in_type != XP_F32 && in_type != XP_BF16) || out_type != XP_F32) return XP_ERR_UNSUPPORTED;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return XP_OK;   // empty output
    if (N == 0 || Cout == 0) return XP_OK;
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    const int64_t K = R * S * Cin;
    if (!output || (K > 0 && (!input || !filter))) return XP_ERR_NULL;
    const int esz = elem_size(in_type);
    if (((uintptr_t)output % 4) != 0 || (K > 0 && (((uintptr_t)input % esz) != 0 || ((uintptr_t)filter % esz) != 0))) return XP_ERR_ALIGN;
    if (H * W > 0x7fffffffLL || P * Q > 0x7fffffffLL || N > 65535 || Cout > 65535) return XP_ERR_SHAPE;   // transpose grids
    const size_t need = xp_conv2d_nchw_workspace_bytes(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, in_type);
    if (is_static && need > workspace_bytes) return XP_ERR_SHAPE;   // beyond the built-in buffer: use the workspace entry point
    if (!workspace || ((uintptr_t)workspace % 256) != 0 || workspace_bytes < need) return XP_ERR_WORKSPACE;

    char *x_nhwc = (char *)workspace;
    char *w_krsc = x_nhwc + round256((size_t)(N * H * W * Cin) * esz);
    hipStream_t s = (hipStream_t)stream;
    if (K > 0) {
        if (transpose(input, x_nhwc, N, Cin, H * W, esz, s) != hipSuccess) return XP_ERR_LAUNCH;        // [N][C][HW] -> [N][HW][C]
        if (transpose(filter, w_krsc, Cout, Cin, R * S, esz, s) != hipSuccess) return XP_ERR_LAUNCH;    // [K][C][RS] -> [K][RS][C]
    }
    Problem q;
    bool nothing;
    const xp_status st = make_conv_problem(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, x_nhwc, in_type,
                                           w_krsc, w_type, XP_FILTER_KRSC, output, XP_F32, stream, &q, &nothing);
    if (st != XP_OK) return st;
    if (nothing) return XP_OK;
    q.c_plane = P * Q;                                    // the kernels' epilogue writes [N][K][PQ] directly
    return run(q);
}

}  // namespace
}  // namespace xp

using namespace xp;

extern "C" {

size_t xp_conv2d_nchw_workspace_bytes(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                                      int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, xp_dtype in_type)
{
    if (N < 0 || H < 0 || W < 0 || Cin < 0 || Cout < 0 || R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 ||
        pad_w < 0 || (in_type != XP_F32 && in_type != XP_BF16))
        return 0;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return 0;
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    const size_t esz = (size_t)elem_size(in_type);
    (void)P; (void)Q;
    return round256((size_t)(N * H * W * Cin) * esz) + round256((size_t)(Cout * R * S * Cin) * esz);
}

xp_status xp_conv2d_nchw(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                         int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                         const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                         void *output, xp_dtype out_type, void *workspace, size_t workspace_bytes, void *stream)
{
    return conv2d_nchw_in(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, input, in_type, filter, w_type, output,
                          out_type, workspace, workspace_bytes, false, stream);
}

size_t xp_conv2d_nchw_static_max_bytes(void) { return STATIC_BYTES; }

xp_status xp_conv2d_nchw_static(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t R, int64_t S,
                                int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                                void *output, xp_dtype out_type, void *stream)
{
    void *ws = nullptr;
    const xp_status st = static_scratch(&ws);
    if (st != XP_OK) return st;
    return conv2d_nchw_in(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, input, in_type, filter, w_type, output,
                          out_type, ws, STATIC_BYTES, true, stream);
}

}  // extern "C"
