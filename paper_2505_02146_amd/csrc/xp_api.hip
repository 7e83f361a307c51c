// Host side of the C ABI declared in include/xp.h: argument validation, canonicalisation of a
// call into xp::Problem, selection of a kernel variant, launch.  No device code lives here.
#include <atomic>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "xp_internal.hpp"

#include <cmath>

namespace xp {

namespace {

constexpr int kMaxVariants = 128;                       // 68 bf16 variants at the last count; checked in build_tables
const Variant *g_table[3][kMaxVariants];
int g_count[3] = {0, 0, 0};
std::once_flag g_once;

int type_slot(xp_dtype t) { return t == XP_F32 ? 0 : (t == XP_BF16 ? 1 : (t == XP_I8 ? 2 : -1)); }

void build_tables()
{
    const xp_dtype types[3] = {XP_F32, XP_BF16, XP_I8};
    for (int s = 0; s < 3; ++s) {
        int n = generic_variants(types[s], g_table[s]);
        if (types[s] == XP_F32) n += f32_mfma_variants(g_table[s] + n);
        else {
            n += kc_variants(types[s], g_table[s] + n);
            n += dl_variants(types[s], g_table[s] + n);
            n += oc_variants(types[s], g_table[s] + n);
            n += sk_variants(types[s], g_table[s] + n);
            n += pp_variants(types[s], g_table[s] + n);
            n += dl_asym_variants(types[s], g_table[s] + n);
        }
        n += gemv_variants(types[s], g_table[s] + n);
        n += dl_bnm_variants(types[s], g_table[s] + n);       // newest last: the older variants keep their indices
        n += dl_asm_variants(types[s], g_table[s] + n);
        n += dl_small_variants(types[s], g_table[s] + n);
        n += rs_variants(types[s], g_table[s] + n);
        if (types[s] == XP_F32) n += f32_small_variants(g_table[s] + n);
        n += dl_pair_variants(types[s], g_table[s] + n);
        if (n > kMaxVariants) { fprintf(stderr, "xp: variant table overflow (%d)\n", n); abort(); }
        g_count[s] = n;
    }
}

// forced variant per (op, type slot); -1 = use the selection table
std::atomic<int> g_forced[4][3];
std::atomic<int> g_last[4][3];
struct Init {
    Init()
    {
        for (auto &r : g_forced) for (auto &x : r) x.store(-1);
        for (auto &r : g_last) for (auto &x : r) x.store(-1);
    }
} g_init;

}  // namespace

int num_variants(xp_dtype in_type)
{
    std::call_once(g_once, build_tables);
    const int s = type_slot(in_type);
    return s < 0 ? 0 : g_count[s];
}

const Variant *variant(xp_dtype in_type, int idx)
{
    std::call_once(g_once, build_tables);
    const int s = type_slot(in_type);
    if (s < 0 || idx < 0 || idx >= g_count[s]) return nullptr;
    return g_table[s][idx];
}

namespace {

// Selection.  Shapes that have been swept on the hardware (sweep.py / tune_grid.py: every variant
// forced, gated and timed -- the brute-force parameter search of Section 5.1 of the paper with the
// reward of Eq. 3-4) are looked up in a table of winners.  The first entries are the workloads, swept
// by hand; xp_tuned_table.inc is a grid of common shapes the run-time tuner went through.  A shape
// that is not in the table takes the winner of its nearest neighbour there -- same operator, type
// and operand contiguity, distance = sum of |log2| of the ratios of batch, M, N and K, at most
// kNear -- since the best tile changes slowly with the shape.  Anything farther from every swept
// shape falls back to a cost estimate that every variant supplies (rounds of workgroups on 256
// compute units x tile work / swept efficiency); the cheapest variant that can run the call wins.
// Variant 0 always can.
struct Tuned {
    xp_op op;
    xp_dtype type;
    int64_t batch, M, N, K;
    bool a_kc, b_kc;            // operand contiguous along K
    const char *variant;
};

const Tuned kTuned[] = {
    {XP_OP_GEMM, XP_F32, 1, 256, 256, 256, true, false, "f32 32x32x256 four waves split k, whole chunk in flight, mfma32x32x2"},
    {XP_OP_GEMM, XP_BF16, 1, 4096, 4096, 4096, true, true, "bf16 256x256x128B waves 2x2 ring 3(A)+2(B) direct-to-lds, reads as assembly, sub-steps paired, mfma16"},
    {XP_OP_GEMM, XP_I8, 1, 4096, 4096, 8192, true, true, "i8 256x256x128B waves 2x2 ring 3(A)+2(B) direct-to-lds, reads as assembly, sub-steps paired, mfma16"},
    {XP_OP_GEMM_BATCHED, XP_BF16, 96, 512, 512, 64, true, true, "bf16 64x128-stream x128B single-k-step producer/consumer nt-stores mfma32"},
    {XP_OP_GEMM_BATCHED, XP_BF16, 96, 512, 64, 512, true, false, "bf16 64x64x128B waves 2x2 k-group-interleaved mfma32"},
    {XP_OP_CONV2D, XP_BF16, 1, 100352, 256, 2304, true, true, "bf16 224x256x128B then 192x256 in the last round, waves 2x2 ring 3(A)+2(B) direct-to-lds, reads as assembly, sub-steps paired, mfma16"},
    // (the same stage with a planar, NCHW, output: the variant above declines it)
    {XP_OP_CONV2D, XP_BF16, 1, 100352, 256, 2304, true, true, "bf16 224x256x128B then 192x256 in the last round, waves 2x4 ring 2(A)+2(B) direct-to-lds, reads as assembly, mfma16"},
#include "xp_tuned_table.inc"
};
constexpr int kNumTuned = (int)(sizeof kTuned / sizeof kTuned[0]);
constexpr float kNear = 2.0f;

// per entry, resolved once: the variant's index and the logarithms of the extents
struct TunedIndex {
    int variant[kNumTuned];
    float lg[kNumTuned][4];
    TunedIndex()
    {
        for (int i = 0; i < kNumTuned; ++i) {
            const Tuned &t = kTuned[i];
            variant[i] = -1;
            const int n = num_variants(t.type);
            for (int v = 0; v < n; ++v)
                if (strcmp(xp::variant(t.type, v)->name, t.variant) == 0) variant[i] = v;
            lg[i][0] = log2f((float)t.batch); lg[i][1] = log2f((float)t.M); lg[i][2] = log2f((float)t.N); lg[i][3] = log2f((float)t.K);
        }
    }
};

int tuned_variant(const Problem &q)
{
    static const TunedIndex index;
    const bool a_kc = q.conv || q.a_sk == 1, b_kc = q.b_sk == 1;
    // an exact entry wins (the first one: the hand-swept workloads precede the grid)
    for (int i = 0; i < kNumTuned; ++i) {
        const Tuned &t = kTuned[i];
        if (t.op == q.op && t.type == q.in_type && t.batch == q.batch && t.M == q.M && t.N == q.N && t.K == q.K && t.a_kc == a_kc &&
            t.b_kc == b_kc) {
            const int v = index.variant[i];
            if (v >= 0 && variant(q.in_type, v)->can_run(q)) return v;
            // (an entry whose variant declines this call -- a planar output, say -- leaves it to a later entry for the shape)
        }
    }
    if (q.K <= 0) return -1;
    const float lq[4] = {log2f((float)q.batch), log2f((float)q.M), log2f((float)q.N), log2f((float)q.K)};
    int best = -1;
    // XP_TABLE_NEAR overrides the radius for tuning experiments (0: exact entries only)
    static const float near = [] { const char *e = getenv("XP_TABLE_NEAR"); return e ? (float)atof(e) : kNear; }();
    float best_d = near;
    for (int i = 0; i < kNumTuned; ++i) {
        const Tuned &t = kTuned[i];
        if (t.op != q.op || t.type != q.in_type || t.a_kc != a_kc || t.b_kc != b_kc || index.variant[i] < 0) continue;
        const float d = fabsf(lq[0] - index.lg[i][0]) + fabsf(lq[1] - index.lg[i][1]) + fabsf(lq[2] - index.lg[i][2]) +
                        fabsf(lq[3] - index.lg[i][3]);
        if (d <= best_d && variant(q.in_type, index.variant[i])->can_run(q)) { best_d = d; best = index.variant[i]; }
    }
    return best;
}

int select_uncached(const Problem &q)
{
    const int learned = runtime_tuned_variant(q);        // shapes tuned in this process or loaded from a file
    if (learned >= 0) return learned;
    const int tuned = tuned_variant(q);
    if (tuned >= 0) return tuned;
    const int n = num_variants(q.in_type);
    int best = 0;
    double best_cost = variant(q.in_type, 0)->cost(q);
    for (int i = 1; i < n; ++i) {
        const Variant *v = variant(q.in_type, i);
        if (!v->can_run(q)) continue;
        const double c = v->cost(q);
        if (c < best_cost) { best_cost = c; best = i; }
    }
    return best;
}

// Programs call the same few shapes over and over, and a table walk costs microseconds that a small
// kernel does not have: each thread remembers its last selections.  A remembered variant is used
// only if it can still run this call (alignment and pitches are not part of the key); changes of the
// run-time table invalidate everything through the generation count.
std::atomic<unsigned> g_generation{1};

struct SelKey {
    int64_t op, type, kc, batch, M, N, K, planar;
    int64_t geom[9];                                      // convolution: H, W, Cin, R, S, strides, pads (the run-time table is keyed on them too)
    bool operator==(const SelKey &o) const { return memcmp(this, &o, sizeof *this) == 0; }
};
struct SelSlot {
    SelKey key;
    int variant;
    unsigned generation;                                  // 0: empty
};

int select_variant(const Problem &q)
{
    constexpr int SLOTS = 64;
    static thread_local SelSlot cache[SLOTS];
    SelKey k;
    k.op = q.op; k.type = q.in_type; k.kc = ((q.conv || q.a_sk == 1) ? 1 : 0) | (q.b_sk == 1 ? 2 : 0);
    k.batch = q.batch; k.M = q.M; k.N = q.N; k.K = q.K; k.planar = q.c_plane != 0;
    const int64_t geom[9] = {q.H, q.W, q.Cin, q.R, q.S, q.sh, q.sw, q.ph, q.pw};
    for (int i = 0; i < 9; ++i) k.geom[i] = q.conv ? geom[i] : 0;
    uint64_t h = 1469598103934665603ull;
    for (const int64_t w : {k.op, k.type, k.kc, k.batch, k.M, k.N, k.K, k.planar}) { h ^= (uint64_t)w; h *= 1099511628211ull; }
    for (const int64_t w : k.geom) { h ^= (uint64_t)w; h *= 1099511628211ull; }
    SelSlot &slot = cache[(h >> 20) % SLOTS];
    const unsigned gen = g_generation.load(std::memory_order_acquire);
    if (slot.generation == gen && slot.key == k) {
        const Variant *v = variant(q.in_type, slot.variant);
        if (v && v->can_run(q)) return slot.variant;
    }
    const int v = select_uncached(q);
    slot.key = k;
    slot.variant = v;
    slot.generation = gen;
    return v;
}

}  // namespace

void selection_changed() { g_generation.fetch_add(1, std::memory_order_acq_rel); }

xp_status launch_variant(const Problem &q, int idx)
{
    const Variant *v = variant(q.in_type, idx);
    if (!v || !v->can_run(q)) return XP_ERR_CONFIG;
    return v->launch(q) == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

xp_status run(const Problem &q)
{
    const int slot = type_slot(q.in_type);
    const int forced = g_forced[q.op][slot].load();
    int idx;
    if (forced >= 0) {
        const Variant *v = variant(q.in_type, forced);
        if (!v || !v->can_run(q)) return XP_ERR_CONFIG;
        idx = forced;
    } else {
        idx = select_variant(q);
    }
    const Variant *v = variant(q.in_type, idx);
    if (!v || !v->can_run(q)) return XP_ERR_UNSUPPORTED;
    g_last[q.op][slot].store(idx);
    return v->launch(q) == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

namespace {

bool aligned_to(const void *p, int bytes) { return ((uintptr_t)p % (uintptr_t)bytes) == 0; }

xp_status check_types(xp_dtype a, xp_dtype b, xp_dtype c, float alpha, float beta)
{
    if (a != b) return XP_ERR_UNSUPPORTED;
    if (a == XP_F32 || a == XP_BF16) return c == XP_F32 ? XP_OK : XP_ERR_UNSUPPORTED;
    if (a == XP_I8) {
        if (c != XP_I32) return XP_ERR_UNSUPPORTED;
        return (alpha == 1.0f && beta == 0.0f) ? XP_OK : XP_ERR_UNSUPPORTED;
    }
    return XP_ERR_UNSUPPORTED;
}

bool bad_layout(int l) { return l != XP_ROW && l != XP_COL; }

}  // namespace

// Validation and canonicalisation of a (batched) GEMM call.  *nothing is set when the call is valid
// but has no output element to compute.
xp_status make_gemm_problem(xp_op op, int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                            const void *A, xp_dtype a_t, xp_layout a_l, int64_t lda, int64_t strideA,
                            const void *B, xp_dtype b_t, xp_layout b_l, int64_t ldb, int64_t strideB,
                            float beta, void *C, xp_dtype c_t, xp_layout c_l, int64_t ldc, int64_t strideC,
                            void *stream, Problem *out, bool *nothing)
{
    *nothing = true;
    if (batch < 0 || M < 0 || N < 0 || K < 0) return XP_ERR_SHAPE;
    if (bad_layout(a_l) || bad_layout(b_l) || bad_layout(c_l)) return XP_ERR_UNSUPPORTED;
    xp_status ts = check_types(a_t, b_t, c_t, alpha, beta);
    if (ts != XP_OK) return ts;
    if (batch == 0 || M == 0 || N == 0) return XP_OK;
    if (!C) return XP_ERR_NULL;
    if (K > 0 && (!A || !B)) return XP_ERR_NULL;
    if (K > 0) {
        if (lda < (a_l == XP_ROW ? K : M)) return XP_ERR_STRIDE;
        if (ldb < (b_l == XP_ROW ? N : K)) return XP_ERR_STRIDE;
    }
    if (ldc < (c_l == XP_ROW ? N : M)) return XP_ERR_STRIDE;
    if (strideA < 0 || strideB < 0 || strideC < 0) return XP_ERR_STRIDE;
    if (batch > 1) {
        const int64_t c_extent = c_l == XP_ROW ? (M - 1) * ldc + N : (N - 1) * ldc + M;
        if (strideC < c_extent) return XP_ERR_STRIDE;
    }
    if (!aligned_to(C, elem_size(c_t)) || (K > 0 && (!aligned_to(A, elem_size(a_t)) || !aligned_to(B, elem_size(b_t)))))
        return XP_ERR_ALIGN;

    Problem q;
    memset(&q, 0, sizeof q);
    q.op = op;
    q.in_type = a_t;
    q.batch = batch;
    q.K = K;
    q.alpha = alpha;
    q.beta = beta;
    q.C = C;
    q.ldc = ldc;
    q.strideA = strideA; q.strideB = strideB; q.strideC = strideC;
    q.conv = false;
    q.stream = (hipStream_t)stream;
    const int64_t a_sm = a_l == XP_ROW ? lda : 1, a_sk = a_l == XP_ROW ? 1 : lda;
    const int64_t b_sk = b_l == XP_ROW ? ldb : 1, b_sn = b_l == XP_ROW ? 1 : ldb;
    if (c_l == XP_ROW) {
        q.M = M; q.N = N;
        q.A = A; q.a_sm = a_sm; q.a_sk = a_sk;
        q.B = B; q.b_sk = b_sk; q.b_sn = b_sn;
    } else {
        // column-major C is the row-major transpose: C^T = B^T . A^T, so the operands trade places
        q.M = N; q.N = M;
        q.A = B; q.a_sm = b_sn; q.a_sk = b_sk;
        q.B = A; q.b_sk = a_sk; q.b_sn = a_sm;
        q.strideA = strideB; q.strideB = strideA;
    }
    if (q.M == 1 && q.N > 1) {
        // a row vector times a matrix is the transposed matrix-vector product: y^T = B^T x^T, with the
        // 1 x N row of C seen as an N x 1 column of unit pitch
        const void *t = q.A; q.A = q.B; q.B = t;
        const int64_t sm = q.b_sn, sk = q.b_sk;
        q.b_sk = q.a_sk; q.b_sn = q.a_sm;
        q.a_sm = sm; q.a_sk = sk;
        const int64_t st = q.strideA; q.strideA = q.strideB; q.strideB = st;
        q.M = q.N; q.N = 1;
        q.ldc = 1;
    }
    *out = q;
    *nothing = false;
    return XP_OK;
}

namespace {

xp_status gemm_common(xp_op op, int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                      const void *A, xp_dtype a_t, xp_layout a_l, int64_t lda, int64_t strideA,
                      const void *B, xp_dtype b_t, xp_layout b_l, int64_t ldb, int64_t strideB,
                      float beta, void *C, xp_dtype c_t, xp_layout c_l, int64_t ldc, int64_t strideC,
                      void *stream)
{
    Problem q;
    bool nothing;
    const xp_status st = make_gemm_problem(op, batch, M, N, K, alpha, A, a_t, a_l, lda, strideA, B, b_t, b_l, ldb, strideB,
                                           beta, C, c_t, c_l, ldc, strideC, stream, &q, &nothing);
    if (st != XP_OK || nothing) return st;
    return run(q);
}

}  // namespace

// Validation and canonicalisation of a convolution call (see make_gemm_problem).
xp_status make_conv_problem(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                            int64_t R, int64_t S, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                            const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                            xp_filter_layout w_layout, void *output, xp_dtype out_type, void *stream,
                            Problem *out, bool *nothing)
{
    *nothing = true;
    if (N < 0 || H < 0 || W < 0 || Cin < 0 || Cout < 0) return XP_ERR_SHAPE;
    if (R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return XP_ERR_SHAPE;
    if (w_layout != XP_FILTER_KRSC && w_layout != XP_FILTER_RSCK) return XP_ERR_UNSUPPORTED;
    if (in_type != w_type || (in_type != XP_F32 && in_type != XP_BF16) || out_type != XP_F32)
        return XP_ERR_UNSUPPORTED;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return XP_OK;   // empty output
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1;
    const int64_t Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N == 0 || Cout == 0) return XP_OK;
    if (!output) return XP_ERR_NULL;
    const int64_t K = R * S * Cin;
    if (K > 0 && (!input || !filter)) return XP_ERR_NULL;
    if (!aligned_to(output, 4) || (K > 0 && (!aligned_to(input, elem_size(in_type)) ||
                                             !aligned_to(filter, elem_size(w_type)))))
        return XP_ERR_ALIGN;

    Problem q;
    memset(&q, 0, sizeof q);
    q.op = XP_OP_CONV2D;
    q.in_type = in_type;
    q.batch = 1;
    q.M = N * P * Q;
    q.N = Cout;
    q.K = K;
    q.A = input;
    q.B = filter;
    q.C = output;
    if (w_layout == XP_FILTER_KRSC) { q.b_sk = 1; q.b_sn = K; }
    else { q.b_sk = Cout; q.b_sn = 1; }
    q.ldc = Cout;
    q.alpha = 1.0f;
    q.beta = 0.0f;
    q.conv = true;
    q.H = H; q.W = W; q.Cin = Cin; q.R = R; q.S = S; q.P = P; q.Q = Q;
    q.sh = stride_h; q.sw = stride_w; q.ph = pad_h; q.pw = pad_w;
    q.stream = (hipStream_t)stream;
    *out = q;
    *nothing = false;
    return XP_OK;
}

}  // namespace xp

using namespace xp;

extern "C" {

xp_status xp_gemm(int64_t M, int64_t N, int64_t K, float alpha,
                  const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda,
                  const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb,
                  float beta, void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc, void *stream)
{
    return gemm_common(XP_OP_GEMM, 1, M, N, K, alpha, A, a_type, a_layout, lda, 0, B, b_type, b_layout, ldb, 0,
                       beta, C, c_type, c_layout, ldc, 0, stream);
}

xp_status xp_gemm_batched(int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                          const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda, int64_t strideA,
                          const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb, int64_t strideB,
                          float beta, void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc, int64_t strideC,
                          void *stream)
{
    return gemm_common(XP_OP_GEMM_BATCHED, batch, M, N, K, alpha, A, a_type, a_layout, lda, strideA,
                       B, b_type, b_layout, ldb, strideB, beta, C, c_type, c_layout, ldc, strideC, stream);
}

xp_status xp_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                         int64_t R, int64_t S, int64_t stride_h, int64_t stride_w,
                         int64_t pad_h, int64_t pad_w,
                         const void *input, xp_dtype in_type,
                         const void *filter, xp_dtype w_type, xp_filter_layout w_layout,
                         void *output, xp_dtype out_type, void *stream)
{
    Problem q;
    bool nothing;
    const xp_status st = make_conv_problem(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, input, in_type,
                                           filter, w_type, w_layout, output, out_type, stream, &q, &nothing);
    if (st != XP_OK || nothing) return st;
    return run(q);
}

xp_status xp_attention(int64_t batch, int64_t Lq, int64_t Lk, int64_t d, int64_t dv, float scale,
                       const void *Q, xp_dtype q_type, int64_t ldq, int64_t strideQ,
                       const void *K, xp_dtype k_type, int64_t ldk, int64_t strideK,
                       const void *V, xp_dtype v_type, int64_t ldv, int64_t strideV,
                       void *O, xp_dtype o_type, int64_t ldo, int64_t strideO,
                       void *stream)
{
    if (batch < 0 || Lq < 0 || Lk < 0 || d < 0 || dv < 0) return XP_ERR_SHAPE;
    if (q_type != k_type || q_type != v_type || (q_type != XP_F32 && q_type != XP_BF16) || o_type != XP_F32)
        return XP_ERR_UNSUPPORTED;
    if (!(scale == scale) || scale - scale != 0.0f) return XP_ERR_UNSUPPORTED;      // NaN or infinite
    if (batch == 0 || Lq == 0 || dv == 0) return XP_OK;
    if (Lk == 0) return XP_ERR_SHAPE;
    if (ldq < d || ldk < d || ldv < dv || ldo < dv) return XP_ERR_STRIDE;
    if (strideQ < 0 || strideK < 0 || strideV < 0 || strideO < 0) return XP_ERR_STRIDE;
    if (batch > 1 && strideO < (Lq - 1) * ldo + dv) return XP_ERR_STRIDE;           // O slices must not overlap
    if (!O || !V || (d > 0 && (!Q || !K))) return XP_ERR_NULL;
    const int esz = elem_size(q_type);
    if (!aligned_to(Q, esz) || !aligned_to(K, esz) || !aligned_to(V, esz) || !aligned_to(O, 4)) return XP_ERR_ALIGN;

    AttnProblem q;
    q.in_type = q_type;
    q.batch = batch; q.Lq = Lq; q.Lk = Lk; q.d = d; q.dv = dv;
    q.scale = scale;
    q.Q = Q; q.K = K; q.V = V; q.O = O;
    q.ldq = ldq; q.ldk = ldk; q.ldv = ldv; q.ldo = ldo;
    q.strideQ = strideQ; q.strideK = strideK; q.strideV = strideV; q.strideO = strideO;
    q.stream = (hipStream_t)stream;

    const int slot = type_slot(q_type);
    const int forced = g_forced[XP_OP_ATTENTION][slot].load();
    int idx = 0;
    if (forced >= 0) {
        const AttnVariant *v = attn_variant(q_type, forced);
        if (!v || !v->can_run(q)) return XP_ERR_CONFIG;
        idx = forced;
    } else {
        // the last variant that can run the call and finds it worthwhile: the table is ordered from general to specialised
        for (int i = attn_num_variants(q_type) - 1; i > 0; --i) {
            const AttnVariant *v = attn_variant(q_type, i);
            if (v->can_run(q) && (!v->worthwhile || v->worthwhile(q))) { idx = i; break; }
        }
    }
    const AttnVariant *v = attn_variant(q_type, idx);
    if (!v || !v->can_run(q)) return XP_ERR_UNSUPPORTED;
    g_last[XP_OP_ATTENTION][slot].store(idx);
    return v->launch(q) == hipSuccess ? XP_OK : XP_ERR_LAUNCH;
}

int xp_num_configs(xp_op op, xp_dtype in_type)
{
    if (op == XP_OP_ATTENTION) return attn_num_variants(in_type);
    if (op < 0 || op > 2) return 0;
    return num_variants(in_type);
}

xp_status xp_describe_config(xp_op op, xp_dtype in_type, int idx, char *buf, size_t n)
{
    if (op < 0 || op > 3 || !buf || n == 0) return XP_ERR_CONFIG;
    if (op == XP_OP_ATTENTION) {
        const AttnVariant *a = attn_variant(in_type, idx);
        if (!a) return XP_ERR_CONFIG;
        snprintf(buf, n, "%s", a->name);
        return XP_OK;
    }
    const Variant *v = variant(in_type, idx);
    if (!v) return XP_ERR_CONFIG;
    snprintf(buf, n, "%s", v->name);
    return XP_OK;
}

xp_status xp_force_config(xp_op op, xp_dtype in_type, int idx)
{
    const int slot = in_type == XP_F32 ? 0 : (in_type == XP_BF16 ? 1 : (in_type == XP_I8 ? 2 : -1));
    if (op < 0 || op > 3 || slot < 0) return XP_ERR_CONFIG;
    if (idx >= (op == XP_OP_ATTENTION ? attn_num_variants(in_type) : num_variants(in_type))) return XP_ERR_CONFIG;
    g_forced[op][slot].store(idx < 0 ? -1 : idx);
    return XP_OK;
}

int xp_last_config(xp_op op, xp_dtype in_type)
{
    const int slot = in_type == XP_F32 ? 0 : (in_type == XP_BF16 ? 1 : (in_type == XP_I8 ? 2 : -1));
    if (op < 0 || op > 3 || slot < 0) return -1;
    return g_last[op][slot].load();
}

const char *xp_status_string(xp_status s)
{
    switch (s) {
    case XP_OK: return "ok";
    case XP_ERR_NULL: return "null pointer for a non-empty operand";
    case XP_ERR_SHAPE: return "invalid extent";
    case XP_ERR_STRIDE: return "leading dimension or batch stride too small";
    case XP_ERR_ALIGN: return "pointer not aligned to its element size";
    case XP_ERR_UNSUPPORTED: return "unsupported dtype, layout or scaling combination";
    case XP_ERR_CONFIG: return "kernel configuration does not exist or cannot run this call";
    case XP_ERR_LAUNCH: return "kernel launch failed";
    case XP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    }
    return "unknown status";
}

const char *xp_version(void) { return "xp 0.1 (gfx950)"; }

}  // extern "C"
