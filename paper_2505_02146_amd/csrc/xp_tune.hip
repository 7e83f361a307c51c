// Run-time parameter search: the brute-force intra-pass auto-tuning of the paper (Section 5.1)
// with its reward (Eq. 3-4: the throughput of a candidate if it is valid, else 0; the best
// candidate wins), and the table of shapes it has tuned.
//
// A candidate is a compiled kernel variant.  Validity is judged on the device against the general
// kernel's result for the same operands: every element finite and a relative Frobenius distance of
// at most 1e-5 (fp32 summation-order noise; a dropped K step or a misplaced tile is 1e-2 or more),
// bit-exact for int8.  The winner is stored under a key made of everything selection depends on,
// by NAME, so that a saved table survives changes of the variant numbering.
#include "xp_internal.hpp"

#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <unordered_map>

namespace xp {
namespace {

std::mutex g_mutex;
std::map<std::string, std::string> g_table;     // shape key -> variant name: what is saved and loaded

// The same table for the launch path, which must not format strings: the key as plain numbers
// (everything shape_key prints), the variant resolved to its index.
struct FastKey {
    int64_t v[16];
    bool operator==(const FastKey &o) const { return memcmp(v, o.v, sizeof v) == 0; }
};
struct FastHash {
    size_t operator()(const FastKey &k) const
    {
        uint64_t h = 1469598103934665603ull;                // FNV-1a over the words
        for (int64_t w : k.v) { h ^= (uint64_t)w; h *= 1099511628211ull; }
        return (size_t)h;
    }
};
std::unordered_map<FastKey, int, FastHash> g_fast;

FastKey fast_key(const Problem &q)
{
    FastKey k;
    memset(&k, 0, sizeof k);
    const int a_kc = (q.conv || q.a_sk == 1) ? 1 : 0, b_kc = q.b_sk == 1 ? 1 : 0;
    k.v[0] = q.conv ? -1 : (int64_t)q.op;
    k.v[1] = (int64_t)q.in_type;
    k.v[2] = b_kc;
    if (q.conv) {
        const int64_t c[] = {q.M / (q.P * q.Q), q.H, q.W, q.Cin, q.N, q.R, q.S, q.sh, q.sw, q.ph, q.pw};
        for (int i = 0; i < 11; ++i) k.v[3 + i] = c[i];
    } else {
        k.v[3] = q.batch; k.v[4] = q.M; k.v[5] = q.N; k.v[6] = q.K; k.v[7] = a_kc;
    }
    return k;
}

// the inverse of shape_key, for tables read from a file; false if the text is not a key
bool parse_key(const char *text, FastKey *k, xp_dtype *type)
{
    memset(k, 0, sizeof *k);
    long long c[12];
    int t, op, a, b;
    if (sscanf(text, "conv t%d n%lld h%lld w%lld c%lld k%lld r%lld s%lld sh%lld sw%lld ph%lld pw%lld b%d", &t, &c[0], &c[1], &c[2],
               &c[3], &c[4], &c[5], &c[6], &c[7], &c[8], &c[9], &c[10], &b) == 13) {
        k->v[0] = -1; k->v[1] = t; k->v[2] = b;
        for (int i = 0; i < 11; ++i) k->v[3 + i] = c[i];
        *type = (xp_dtype)t;
        return true;
    }
    if (sscanf(text, "gemm%d t%d b%lld m%lld n%lld k%lld a%d b%d", &op, &t, &c[0], &c[1], &c[2], &c[3], &a, &b) == 8) {
        k->v[0] = op; k->v[1] = t; k->v[2] = b; k->v[3] = c[0]; k->v[4] = c[1]; k->v[5] = c[2]; k->v[6] = c[3]; k->v[7] = a;
        *type = (xp_dtype)t;
        return true;
    }
    return false;
}

std::string shape_key(const Problem &q)
{
    char buf[256];
    const int a_kc = (q.conv || q.a_sk == 1) ? 1 : 0, b_kc = q.b_sk == 1 ? 1 : 0;
    if (q.conv)
        snprintf(buf, sizeof buf, "conv t%d n%lld h%lld w%lld c%lld k%lld r%lld s%lld sh%lld sw%lld ph%lld pw%lld b%d",
                 (int)q.in_type, (long long)(q.M / (q.P * q.Q)), (long long)q.H, (long long)q.W, (long long)q.Cin,
                 (long long)q.N, (long long)q.R, (long long)q.S, (long long)q.sh, (long long)q.sw, (long long)q.ph,
                 (long long)q.pw, b_kc);
    else
        snprintf(buf, sizeof buf, "gemm%d t%d b%lld m%lld n%lld k%lld a%d b%d", (int)q.op, (int)q.in_type,
                 (long long)q.batch, (long long)q.M, (long long)q.N, (long long)q.K, a_kc, b_kc);
    return buf;
}

int variant_by_name(xp_dtype t, const std::string &name)
{
    const int n = num_variants(t);
    for (int i = 0; i < n; ++i)
        if (name == variant(t, i)->name) return i;
    return -1;
}

// ---- device side: comparison of a candidate with the reference
// out[0] = sum (cand - ref)^2, out[1] = sum ref^2, out[2] = number of non-finite candidate elements
// (int: out[0] = number of differing elements).  One workgroup: the tuner is not on a critical path,
// and a single pass in a fixed order keeps the verdict deterministic.
struct CmpParams {
    const void *ref, *cand;
    long long batch, M, N, ldc, strideC;
    double *out;
};

template <bool INT>
__global__ __launch_bounds__(1024) void compare_kernel(CmpParams p)
{
    __shared__ double red[3][1024];
    const int t = threadIdx.x;
    double d2 = 0.0, r2 = 0.0, bad = 0.0;
    const long long per = p.M * p.N, total = p.batch * per;
    for (long long e = t; e < total; e += 1024) {
        const long long b = e / per, rest = e % per;
        const long long off = b * p.strideC + (rest / p.N) * p.ldc + rest % p.N;
        if constexpr (INT) {
            if (((const int *)p.ref)[off] != ((const int *)p.cand)[off]) d2 += 1.0;
        } else {
            const float r = ((const float *)p.ref)[off], c = ((const float *)p.cand)[off];
            if (!(c - c == 0.0f)) bad += 1.0;            // NaN or infinity
            else {
                const double d = (double)c - (double)r;
                d2 += d * d;
            }
            r2 += (double)r * (double)r;
        }
    }
    red[0][t] = d2; red[1][t] = r2; red[2][t] = bad;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (t < s)
            for (int k = 0; k < 3; ++k) red[k][t] += red[k][t + s];
        __syncthreads();
    }
    if (t < 3) p.out[t] = red[t][0];
}

size_t round256(size_t x) { return (x + 255) / 256 * 256; }

int64_t c_extent(const Problem &q) { return (q.batch - 1) * q.strideC + (q.M - 1) * q.ldc + q.N; }

xp_status tune(const Problem &q0, void *workspace, size_t workspace_bytes, int reps, int *best, float *best_us)
{
    if (reps < 1) return XP_ERR_SHAPE;
    const size_t bytes = (size_t)c_extent(q0) * 4;
    if (!workspace || ((uintptr_t)workspace % 256) != 0 || workspace_bytes < 2 * round256(bytes) + 256) return XP_ERR_WORKSPACE;
    char *ref = (char *)workspace, *cand = ref + round256(bytes);
    double *stats = (double *)(cand + round256(bytes));
    hipStream_t stream = q0.stream;
    const bool is_int = q0.in_type == XP_I8;

    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return XP_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return XP_ERR_LAUNCH; }
    auto fail = [&](xp_status st) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return st; };

    // the reference: the general kernel on a copy of C
    Problem q = q0;
    if (hipMemcpyAsync(ref, q0.C, bytes, hipMemcpyDeviceToDevice, stream) != hipSuccess) return fail(XP_ERR_LAUNCH);
    q.C = ref;
    xp_status st = launch_variant(q, 0);
    if (st != XP_OK) return fail(st);

    CmpParams cp;
    cp.ref = ref; cp.cand = cand; cp.batch = q0.batch; cp.M = q0.M; cp.N = q0.N; cp.ldc = q0.ldc; cp.strideC = q0.strideC;
    cp.out = stats;

    auto time_variant = [&](int v, float *us) {
        (void)hipEventRecord(e0, stream);
        for (int i = 0; i < reps; ++i)
            if (launch_variant(q, v) != XP_OK) return false;
        (void)hipEventRecord(e1, stream);
        if (hipEventSynchronize(e1) != hipSuccess) return false;
        float ms = 0.0f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        *us = ms * 1e3f / (float)reps;
        return true;
    };

    // first pass: every candidate once; the three fastest go on to the second pass
    constexpr int TOP = 3;
    int top_v[TOP] = {-1, -1, -1};
    float top_us[TOP] = {0.0f, 0.0f, 0.0f};
    const int n = num_variants(q0.in_type);
    for (int v = 0; v < n; ++v) {
        q.C = cand;
        if (!variant(q0.in_type, v)->can_run(q)) continue;                         // reward 0: not a candidate
        if (hipMemcpyAsync(cand, q0.C, bytes, hipMemcpyDeviceToDevice, stream) != hipSuccess) return fail(XP_ERR_LAUNCH);
        if (launch_variant(q, v) != XP_OK) continue;
        if (is_int) hipLaunchKernelGGL(compare_kernel<true>, dim3(1), dim3(1024), 0, stream, cp);
        else hipLaunchKernelGGL(compare_kernel<false>, dim3(1), dim3(1024), 0, stream, cp);
        double h[3] = {1.0, 0.0, 1.0};
        if (hipMemcpyAsync(h, stats, sizeof h, hipMemcpyDeviceToHost, stream) != hipSuccess) return fail(XP_ERR_LAUNCH);
        if (hipStreamSynchronize(stream) != hipSuccess) return fail(XP_ERR_LAUNCH);
        const bool valid = is_int ? h[0] == 0.0 : (h[2] == 0.0 && h[0] <= 1e-10 * h[1]);   // (1e-5)^2 on the squares
        if (!valid) continue;                                                      // reward 0
        for (int i = 0; i < 2; ++i)
            if (launch_variant(q, v) != XP_OK) return fail(XP_ERR_LAUNCH);
        float us;
        if (!time_variant(v, &us)) return fail(XP_ERR_LAUNCH);
        for (int k = 0; k < TOP; ++k) {                                            // insertion into the sorted top list
            if (top_v[k] < 0 || us < top_us[k]) {
                for (int j = TOP - 1; j > k; --j) { top_v[j] = top_v[j - 1]; top_us[j] = top_us[j - 1]; }
                top_v[k] = v;
                top_us[k] = us;
                break;
            }
        }
    }
    // second pass: the finalists again, in turn, twice; each keeps its best time (clocks drift
    // under the power limit, so neighbours in time are the fair comparison)
    // The second pass runs each finalist for about 5 ms at a time: under sustained load the chip sits at
    // its power limit and a variant that draws less for the same work clocks higher -- a burst of a few
    // launches ranks such variants differently from the way a program that keeps calling them sees them.
    const int reps1 = reps;
    if (top_v[0] >= 0 && top_us[0] > 0.0f) {
        const float want = 5000.0f / top_us[0];
        reps = want > 1000.0f ? 1000 : (want > (float)reps1 ? (int)want : reps1);
    }
    for (int k = 0; k < TOP; ++k) top_us[k] = 0.0f;
    for (int round = 0; round < 2; ++round)
        for (int k = 0; k < TOP; ++k) {
            if (top_v[k] < 0) continue;
            float us;
            if (!time_variant(top_v[k], &us)) return fail(XP_ERR_LAUNCH);
            if (top_us[k] == 0.0f || us < top_us[k]) top_us[k] = us;
        }
    int win = 0;
    float win_us = 0.0f;
    for (int k = 0; k < TOP; ++k)
        if (top_v[k] >= 0 && (win_us == 0.0f || top_us[k] < win_us)) { win = top_v[k]; win_us = top_us[k]; }   // largest reward
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (win_us == 0.0f) return XP_ERR_UNSUPPORTED;                                  // not even the general kernel ran
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        g_table[shape_key(q0)] = variant(q0.in_type, win)->name;
        g_fast[fast_key(q0)] = win;
    }
    selection_changed();
    if (best) *best = win;
    if (best_us) *best_us = win_us;
    return launch_variant(q0, win);                                                 // C itself, once, with the winner
}

}  // namespace

int runtime_tuned_variant(const Problem &q)
{
    int v;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        if (g_fast.empty()) return -1;
        auto it = g_fast.find(fast_key(q));
        if (it == g_fast.end()) return -1;
        v = it->second;
    }
    return variant(q.in_type, v)->can_run(q) ? v : -1;
}

}  // namespace xp

using namespace xp;

extern "C" {

xp_status xp_tune_gemm(int64_t M, int64_t N, int64_t K, float alpha,
                       const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda,
                       const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb,
                       float beta, void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc,
                       void *workspace, size_t workspace_bytes, int reps, int *best, float *best_us, void *stream)
{
    Problem q;
    bool nothing;
    const xp_status st = make_gemm_problem(XP_OP_GEMM, 1, M, N, K, alpha, A, a_type, a_layout, lda, 0, B, b_type, b_layout,
                                           ldb, 0, beta, C, c_type, c_layout, ldc, 0, stream, &q, &nothing);
    if (st != XP_OK || nothing) return st;
    if (q.K == 0) return run(q);
    return tune(q, workspace, workspace_bytes, reps, best, best_us);
}

xp_status xp_tune_gemm_batched(int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                               const void *A, xp_dtype a_type, xp_layout a_layout, int64_t lda, int64_t strideA,
                               const void *B, xp_dtype b_type, xp_layout b_layout, int64_t ldb, int64_t strideB,
                               float beta, void *C, xp_dtype c_type, xp_layout c_layout, int64_t ldc, int64_t strideC,
                               void *workspace, size_t workspace_bytes, int reps, int *best, float *best_us, void *stream)
{
    Problem q;
    bool nothing;
    const xp_status st = make_gemm_problem(XP_OP_GEMM_BATCHED, batch, M, N, K, alpha, A, a_type, a_layout, lda, strideA,
                                           B, b_type, b_layout, ldb, strideB, beta, C, c_type, c_layout, ldc, strideC,
                                           stream, &q, &nothing);
    if (st != XP_OK || nothing) return st;
    if (q.K == 0) return run(q);
    return tune(q, workspace, workspace_bytes, reps, best, best_us);
}

xp_status xp_tune_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                              int64_t R, int64_t S, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                              const void *input, xp_dtype in_type, const void *filter, xp_dtype w_type,
                              xp_filter_layout w_layout, void *output, xp_dtype out_type,
                              void *workspace, size_t workspace_bytes, int reps, int *best, float *best_us, void *stream)
{
    Problem q;
    bool nothing;
    const xp_status st = make_conv_problem(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, input, in_type,
                                           filter, w_type, w_layout, output, out_type, stream, &q, &nothing);
    if (st != XP_OK || nothing) return st;
    if (q.K == 0) return run(q);
    return tune(q, workspace, workspace_bytes, reps, best, best_us);
}

size_t xp_tune_workspace_bytes(int64_t c_extent_elems)
{
    if (c_extent_elems < 0) return 0;
    return 2 * round256((size_t)c_extent_elems * 4) + 256;
}

xp_status xp_tune_save(const char *path)
{
    if (!path) return XP_ERR_NULL;
    FILE *f = fopen(path, "w");
    if (!f) return XP_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_mutex);
    fprintf(f, "# xp tuned shapes: <shape key> | <variant name>\n");
    for (const auto &kv : g_table) fprintf(f, "%s | %s\n", kv.first.c_str(), kv.second.c_str());
    return fclose(f) == 0 ? XP_OK : XP_ERR_WORKSPACE;
}

xp_status xp_tune_load(const char *path)
{
    if (!path) return XP_ERR_NULL;
    FILE *f = fopen(path, "r");
    if (!f) return XP_ERR_WORKSPACE;
    char line[1024];
    std::lock_guard<std::mutex> lock(g_mutex);
    while (fgets(line, sizeof line, f)) {
        if (line[0] == '#') continue;
        char *bar = strstr(line, " | ");
        if (!bar) continue;
        std::string key(line, bar - line), name(bar + 3);
        while (!name.empty() && (name.back() == '\n' || name.back() == '\r' || name.back() == ' ')) name.pop_back();
        if (key.empty() || name.empty()) continue;
        g_table[key] = name;
        FastKey fk;
        xp_dtype type;
        if (parse_key(key.c_str(), &fk, &type)) {
            const int v = variant_by_name(type, name);       // names this build does not know are kept in the text only
            if (v >= 0) g_fast[fk] = v;
            else g_fast.erase(fk);
        }
    }
    fclose(f);
    selection_changed();
    return XP_OK;
}

void xp_tune_clear(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_table.clear();
    g_fast.clear();
    selection_changed();
}

int xp_tune_count(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    return (int)g_table.size();
}

}  // extern "C"
