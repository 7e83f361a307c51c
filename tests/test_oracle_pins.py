"""Pins for the CPU oracle: closed forms, invariants, hand-computed cases and brute force.

The paper lists GEMM, Batch GEMM and Conv2D NHWC by name only (Table 5) and prints no worked
example, so the oracle is pinned by what mathematics fixes.  Each test is chosen so that one
plausible mistake (wrong index, transposed operand, dropped term, sign of the padding
offset, u8-vs-s8) fails it.  None of them re-types the oracle's loop.
"""
import pathlib

import numpy as np
import pytest

from paper_2505_02146_amd import inputs

GOLDEN = pathlib.Path(__file__).parent / "golden" / "tiny_cases.txt"


def _golden():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        line = line.split("#")[0].strip()
        if "=" not in line:
            continue
        k, v = line.split("=")
        out[k.strip()] = np.array([[float(t) for t in row.split()] for row in v.split(";")])
    return out


def _store(mat: np.ndarray, layout: str, ld_pad: int = 0, fill=np.nan):
    """Flat buffer holding logical matrix `mat` in `layout` with padded leading dimension."""
    rows, cols = mat.shape
    if layout == "row":
        ld = cols + ld_pad
        buf = np.full((rows, ld), fill, dtype=mat.dtype)
        buf[:, :cols] = mat
    else:
        ld = rows + ld_pad
        buf = np.full((cols, ld), fill, dtype=mat.dtype)
        buf[:, :rows] = mat.T
    return np.ascontiguousarray(buf).reshape(-1), ld


LAYOUTS = [("row", "row"), ("row", "col"), ("col", "row"), ("col", "col")]


# ---------------------------------------------------------------- hand-computed cases
def test_golden_gemm(oracle):
    g = _golden()
    A = g["gemm_A"].astype(np.float32)
    B = g["gemm_B"].astype(np.float32)
    for la, lb in LAYOUTS:
        a, lda = _store(A, la, 2, 99.0)
        b, ldb = _store(B, lb, 1, 99.0)
        ref = oracle.gemm_float(2, 2, 3, a, la, b, lb, lda=lda, ldb=ldb)
        assert np.array_equal(ref, g["gemm_C"]), (la, lb)
    for lc in ("row", "col"):
        c0, ldc = _store(np.ones((2, 2), np.float32), lc, 3, 99.0)
        ref = oracle.gemm_float(2, 2, 3, A.reshape(-1), "row", B.reshape(-1), "row",
                                alpha=2.0, beta=3.0, C0=c0, c_layout=lc, ldc=ldc)
        assert np.array_equal(ref, g["gemm_C_alpha2_beta3"])


def test_golden_conv(oracle):
    g = _golden()
    x = g["conv_in"].astype(np.float32).reshape(1, 3, 3, 1)
    w = g["conv_w"].astype(np.float32).reshape(1, 3, 3, 1)
    kw = dict(N=1, H=3, W=3, Cin=1, Cout=1, R=3, S=3)
    ref = oracle.conv2d_nhwc(x, w, pad=(1, 1), **kw)
    assert np.array_equal(ref.reshape(3, 3), g["conv_out"])
    ref = oracle.conv2d_nhwc(x, w, pad=(0, 0), **kw)
    assert ref.shape == (1, 1, 1, 1) and ref.reshape(-1)[0] == g["conv_out_pad0"][0, 0]
    ref = oracle.conv2d_nhwc(x, w, pad=(1, 1), stride=(2, 2), **kw)
    assert np.array_equal(ref.reshape(2, 2), g["conv_out_stride2"])


# ---------------------------------------------------------------- GEMM closed forms
@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_identity_and_padded_ld(oracle, la, lb):
    M, K = 7, 5
    A = inputs.uniform_pm1((M, K), 3, 1)
    a, lda = _store(A, la, 3)
    eye, ldb = _store(np.eye(K, dtype=np.float32), lb, 2)
    ref = oracle.gemm_float(M, K, K, a, la, eye, lb, lda=lda, ldb=ldb)
    assert np.array_equal(ref, A.astype(np.float64))
    eye, lde = _store(np.eye(M, dtype=np.float32), la, 1)
    Bm = inputs.uniform_pm1((M, K), 3, 2)                 # I(MxM) . B(MxK)
    b, ldb = _store(Bm, lb, 4)
    ref = oracle.gemm_float(M, K, M, eye, la, b, lb, lda=lde, ldb=ldb)
    assert np.array_equal(ref, Bm.astype(np.float64))


@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_permutation(oracle, la, lb):
    M, K, N = 6, 6, 4
    perm = np.array([3, 0, 5, 1, 2, 4])
    Pm = np.zeros((M, K), np.float32)
    Pm[np.arange(M), perm] = 1.0                          # (P.B)[i] = B[perm[i]]
    B = inputs.uniform_pm1((K, N), 5, 2)
    a, lda = _store(Pm, la)
    b, ldb = _store(B, lb)
    ref = oracle.gemm_float(M, N, K, a, la, b, lb, lda=lda, ldb=ldb)
    assert np.array_equal(ref, B[perm].astype(np.float64))
    A = inputs.uniform_pm1((N, M), 5, 1)                  # (A.P)[:, perm[i]] = A[:, i]
    a, lda = _store(A, la)
    p, ldp = _store(Pm, lb)
    ref = oracle.gemm_float(N, K, M, a, la, p, lb, lda=lda, ldb=ldp)
    want = np.zeros((N, K))
    want[:, perm] = A
    assert np.array_equal(ref, want)


def test_all_ones_gives_K(oracle):
    for M, N, K in [(3, 4, 1), (5, 2, 17), (2, 2, 1000)]:
        ref = oracle.gemm_float(M, N, K, np.ones(M * K, np.float32), "row",
                                np.ones(K * N, np.float32), "col")
        assert np.array_equal(ref, np.full((M, N), float(K)))


def test_rank_one(oracle):
    u = np.array([1, -2, 3, 0.5], np.float32)
    v = np.array([2, 4, -8], np.float32)
    ref = oracle.gemm_float(4, 3, 1, u, "row", v, "row")
    assert np.array_equal(ref, np.outer(u, v).astype(np.float64))
    K = 9
    A = np.repeat(u[:, None], K, 1).copy().reshape(-1)
    B = np.repeat(v[None, :], K, 0).copy().reshape(-1)
    ref = oracle.gemm_float(4, 3, K, A, "row", B, "row")
    assert np.array_equal(ref, K * np.outer(u, v).astype(np.float64))
    # operand roles: a non-square rank-1 product is not symmetric
    assert not np.array_equal(ref[:3, :3], ref[:3, :3].T)


def test_transpose_identity_bitwise(oracle):
    # (A.B)^T = B^T.A^T; handing the same buffers over with swapped roles and layouts keeps
    # the k order, so the bits agree.
    M, N, K = 5, 7, 11
    A = inputs.uniform_pm1((M, K), 7, 1).reshape(-1)
    B = inputs.uniform_pm1((K, N), 7, 2).reshape(-1)
    ab = oracle.gemm_float(M, N, K, A, "row", B, "row")
    bt_at = oracle.gemm_float(N, M, K, B, "col", A, "col", lda=N, ldb=K)
    assert np.array_equal(ab.T, bt_at)


def test_alpha_beta_and_beta_zero_ignores_c(oracle):
    M, N, K = 4, 5, 6
    A = inputs.small_integers((M, K), 1, 1)
    B = inputs.small_integers((K, N), 1, 2)
    C0 = inputs.small_integers((M, N), 1, 3)
    want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) + 3 * C0.astype(np.int64)
    ref = oracle.gemm_float(M, N, K, A.reshape(-1), "row", B.reshape(-1), "row",
                            alpha=2, beta=3, C0=C0.reshape(-1))
    assert np.array_equal(ref, want.astype(np.float64))
    nan = np.full(M * N, np.nan, np.float32)
    ref = oracle.gemm_float(M, N, K, A.reshape(-1), "row", B.reshape(-1), "row",
                            alpha=1, beta=0, C0=nan)
    assert np.array_equal(ref, (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64))


@pytest.mark.parametrize("la,lb", LAYOUTS)
@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_integer_valued_floats_vs_int64(oracle, la, lb, kind):
    # integer entries in [-8, 8] are exact in bf16 and fp32; numpy's int64 matmul is the truth
    M, N, K = 13, 9, 37
    A = inputs.small_integers((M, K), 11, 1)
    B = inputs.small_integers((K, N), 11, 2)
    want = A.astype(np.int64) @ B.astype(np.int64)
    conv = (lambda x: x) if kind == "f32" else inputs.to_bf16_bits
    a, lda = _store(conv(A).reshape(M, K), la, 1, 0)
    b, ldb = _store(conv(B).reshape(K, N), lb, 2, 0)
    ref = oracle.gemm_float(M, N, K, a, la, b, lb, lda=lda, ldb=ldb)
    assert np.array_equal(ref, want.astype(np.float64))


def test_bf16_widening_is_exact(oracle):
    # 1 x 1 x 1 products of chosen bf16 bit patterns: 0x3FC0 = 1.5, 0xC020 = -2.5, 0x0001 = 2^-133
    cases = [(0x3FC0, 0x3F80, 1.5), (0xC020, 0x3FC0, -3.75), (0x0001, 0x3F80, 2.0 ** -133)]
    for a, b, want in cases:
        ref = oracle.gemm_float(1, 1, 1, np.array([a], np.uint16), "row", np.array([b], np.uint16), "row")
        assert ref[0, 0] == want


def test_fp64_accumulation_not_fp32(oracle):
    # 2^24 + 1 - 2^24 = 1 in fp64, 0 if the sum were kept in fp32
    A = np.array([2.0 ** 24, 1.0, -(2.0 ** 24)], np.float32)
    B = np.ones(3, np.float32)
    assert oracle.gemm_float(1, 1, 3, A, "row", B, "row")[0, 0] == 1.0


def test_random_vs_numpy_float64(oracle):
    # library matmul in fp64 agrees to rounding (different summation order allowed)
    M, N, K = 33, 29, 129
    A = inputs.uniform_pm1((M, K), 2, 1)
    B = inputs.uniform_pm1((K, N), 2, 2)
    ref = oracle.gemm_float(M, N, K, A.reshape(-1), "row", B.reshape(-1), "row")
    want = A.astype(np.float64) @ B.astype(np.float64)
    assert np.max(np.abs(ref - want)) <= 1e-13 * K


def test_degenerate_sizes(oracle):
    z = np.zeros(0, np.float32)
    assert oracle.gemm_float(0, 3, 2, z, "row", np.ones(6, np.float32), "row").shape == (0, 3)
    assert oracle.gemm_float(3, 0, 2, np.ones(6, np.float32), "row", z, "row").shape == (3, 0)
    ref = oracle.gemm_float(2, 2, 0, z, "row", z, "row", beta=2.0, C0=np.array([1, 2, 3, 4], np.float32))
    assert np.array_equal(ref, [[2, 4], [6, 8]])


# ---------------------------------------------------------------- int8
def test_int8_extremes(oracle):
    K = 8192
    lo = np.full(K, -128, np.int8)
    hi = np.full(K, 127, np.int8)
    assert oracle.gemm_i8(1, 1, K, lo, "row", lo, "col")[0, 0] == 2 ** 27 == 134217728
    assert oracle.gemm_i8(1, 1, K, lo, "row", hi, "col")[0, 0] == -133169152   # signed x signed
    assert oracle.gemm_i8(1, 1, K, hi, "row", lo, "col")[0, 0] == -133169152


def test_int8_overflow_detected(oracle):
    K = 1 << 17                                      # 2^17 * 2^14 = 2^31 > INT32_MAX
    lo = np.full(K, -128, np.int8)
    with pytest.raises(OverflowError):
        oracle.gemm_i8(1, 1, K, lo, "row", lo, "col")


@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_int8_vs_numpy_int64(oracle, la, lb):
    M, N, K = 17, 19, 130
    A = inputs.int8_uniform((M, K), 4, 1)
    B = inputs.int8_uniform((K, N), 4, 2)
    a, lda = _store(A, la, 3, 0)
    b, ldb = _store(B, lb, 5, 0)
    ref = oracle.gemm_i8(M, N, K, a, la, b, lb, lda=lda, ldb=ldb)
    assert np.array_equal(ref, A.astype(np.int64) @ B.astype(np.int64))


# ---------------------------------------------------------------- batched
def test_batched_is_loop_of_single(oracle):
    b, M, N, K = 3, 4, 5, 6
    sA, sB = M * K + 7, K * N + 3
    A = inputs.uniform_pm1((b * sA,), 9, 1)
    B = inputs.uniform_pm1((b * sB,), 9, 2)
    ref = oracle.gemm_float_batched(b, M, N, K, A, "row", B, "col", strideA=sA, strideB=sB)
    for i in range(b):
        one = oracle.gemm_float(M, N, K, A[i * sA:i * sA + M * K].copy(), "row",
                                B[i * sB:i * sB + K * N].copy(), "col")
        assert np.array_equal(ref[i], one)
    # and against int64 truth with per-batch distinct integer data and beta
    Ai = inputs.small_integers((b, M, K), 9, 1)
    Bi = inputs.small_integers((b, K, N), 9, 2)
    Ci = inputs.small_integers((b, M, N), 9, 3)
    ref = oracle.gemm_float_batched(b, M, N, K, Ai, "row", Bi, "row", alpha=-1, beta=2, C0=Ci)
    want = -np.einsum("bmk,bkn->bmn", Ai.astype(np.int64), Bi.astype(np.int64)) + 2 * Ci.astype(np.int64)
    assert np.array_equal(ref, want.astype(np.float64))


# ---------------------------------------------------------------- convolution
def _brute_conv_gather(x, w_krsc, stride, pad):
    """Second, independently written direct convolution: pad the image explicitly and take
    strided windows (gather over output positions, tap loops outermost)."""
    N, H, W, Cin = x.shape
    Cout, R, S, _ = w_krsc.shape
    xp = np.zeros((N, H + 2 * pad[0], W + 2 * pad[1], Cin), np.float64)
    xp[:, pad[0]:pad[0] + H, pad[1]:pad[1] + W] = x
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    out = np.zeros((N, P, Q, Cout), np.float64)
    for s in range(S - 1, -1, -1):
        for r in range(R):
            win = xp[:, r:r + (P - 1) * stride[0] + 1:stride[0], s:s + (Q - 1) * stride[1] + 1:stride[1]]
            out += np.einsum("npqc,kc->npqk", win, w_krsc[:, r, s, :].astype(np.float64))
    return out


def test_conv_delta_reproduces_input(oracle):
    N, H, W, C = 2, 5, 4, 3
    x = inputs.uniform_pm1((N, H, W, C), 1, 1)
    w = np.zeros((C, 3, 3, C), np.float32)
    w[np.arange(C), 1, 1, np.arange(C)] = 1.0
    ref = oracle.conv2d_nhwc(x, w, N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, pad=(1, 1))
    assert np.array_equal(ref, x.astype(np.float64))


def test_conv_shifted_delta_is_correlation(oracle):
    N, H, W, C = 1, 4, 5, 2
    x = inputs.uniform_pm1((N, H, W, C), 1, 1)
    w = np.zeros((C, 3, 3, C), np.float32)
    w[np.arange(C), 0, 0, np.arange(C)] = 1.0       # tap (0,0): out[p,q] = in[p-1, q-1]
    ref = oracle.conv2d_nhwc(x, w, N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, pad=(1, 1))
    want = np.zeros_like(ref)
    want[:, 1:, 1:] = x[:, :-1, :-1]
    assert np.array_equal(ref, want)
    w[:] = 0
    w[np.arange(C), 2, 1, np.arange(C)] = 1.0       # tap (2,1): out[p,q] = in[p+1, q]
    ref = oracle.conv2d_nhwc(x, w, N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, pad=(1, 1))
    want[:] = 0
    want[:, :-1, :] = x[:, 1:, :]
    assert np.array_equal(ref, want)


def test_conv_all_ones_counts_valid_taps(oracle):
    N, H, W, Cin, Cout = 1, 5, 6, 4, 2
    x = np.ones((N, H, W, Cin), np.float32)
    w = np.ones((Cout, 3, 3, Cin), np.float32)
    ref = oracle.conv2d_nhwc(x, w, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=3, S=3, pad=(1, 1))
    assert np.all(ref[0, 1:-1, 1:-1] == 9 * Cin)
    assert np.all(ref[0, 0, 1:-1] == 6 * Cin) and np.all(ref[0, 1:-1, -1] == 6 * Cin)
    for p, q in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(ref[0, p, q] == 4 * Cin)


def test_conv_1x1_equals_gemm(oracle):
    N, H, W, Cin, Cout = 2, 3, 4, 5, 6
    x = inputs.uniform_pm1((N, H, W, Cin), 2, 1)
    w = inputs.uniform_pm1((Cout, 1, 1, Cin), 2, 2)
    ref = oracle.conv2d_nhwc(x, w, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=1, S=1)
    g = oracle.gemm_float(N * H * W, Cout, Cin, x.reshape(-1), "row", w.reshape(-1), "col")
    assert np.array_equal(ref.reshape(N * H * W, Cout), g)


def test_conv_equals_explicit_im2col_gemm(oracle):
    # the implicit-GEMM index map m=(n,p,q), k=(r,s,c), written out as a materialised matrix
    N, H, W, Cin, Cout, R, S = 2, 5, 4, 3, 4, 3, 3
    x = inputs.to_bf16_bits(inputs.uniform_pm1((N, H, W, Cin), 6, 1))
    w = inputs.to_bf16_bits(inputs.uniform_pm1((Cout, R, S, Cin), 6, 2))
    ref = oracle.conv2d_nhwc(x, w, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S, pad=(1, 1))
    cols = np.zeros((N * H * W, R * S * Cin), np.uint16)
    for n in range(N):
        for p in range(H):
            for q in range(W):
                for r in range(R):
                    for s in range(S):
                        h, ww = p + r - 1, q + s - 1
                        if 0 <= h < H and 0 <= ww < W:
                            cols[(n * H + p) * W + q, (r * S + s) * Cin:(r * S + s + 1) * Cin] = x[n, h, ww]
    g = oracle.gemm_float(N * H * W, Cout, R * S * Cin, cols.reshape(-1), "row", w.reshape(-1), "col")
    assert np.array_equal(ref.reshape(N * H * W, Cout), g)


@pytest.mark.parametrize("stride,pad,H,W,R,S", [((2, 2), (0, 0), 7, 6, 3, 2), ((1, 2), (2, 1), 5, 8, 2, 3),
                                                ((3, 1), (1, 0), 9, 4, 3, 1), ((1, 1), (1, 1), 4, 4, 3, 3)])
@pytest.mark.parametrize("fl", ["krsc", "rsck"])
def test_conv_general_vs_second_brute_force(oracle, stride, pad, H, W, R, S, fl):
    N, Cin, Cout = 2, 3, 5
    x = inputs.small_integers((N, H, W, Cin), 8, 1)
    w = inputs.small_integers((Cout, R, S, Cin), 8, 2)
    want = _brute_conv_gather(x, w, stride, pad)
    wbuf = w if fl == "krsc" else np.ascontiguousarray(w.transpose(1, 2, 3, 0))
    ref = oracle.conv2d_nhwc(x, wbuf, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S,
                             stride=stride, pad=pad, filter_layout=fl)
    assert ref.shape == want.shape
    assert np.array_equal(ref, want)


def test_conv_empty_output(oracle):
    x = np.ones((1, 2, 2, 1), np.float32)
    w = np.ones((1, 3, 3, 1), np.float32)
    ref = oracle.conv2d_nhwc(x, w, N=1, H=2, W=2, Cin=1, Cout=1, R=3, S=3)
    assert ref.size == 0
