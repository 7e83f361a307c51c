"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Gates: int8 -> int32 results bit-exact; floating point elementwise |err| <= 1e-2 (|ref| + 1) and
relative Frobenius error <= 5e-3, plus the tighter fp32-accumulation bound in helpers.py, plus
bit-exactness on integer-valued inputs (every partial sum exactly representable in fp32).
Every kernel variant is forced in turn, then the library's own selection is checked.
"""
import numpy as np
import pytest

from paper_2505_02146_amd import inputs
from tests.helpers import check_float, dev, store, unstore

pytestmark = pytest.mark.gpu

LAYOUTS = [("row", "col"), ("row", "row"), ("col", "row"), ("col", "col")]
# sizes: single element, below one MFMA block, around tile edges, several 256-tiles with ragged tails
SHAPES = [(1, 1, 1), (15, 17, 16), (33, 31, 8), (63, 65, 64), (129, 255, 72), (257, 130, 200), (300, 520, 328),
          (264, 136, 200), (272, 144, 203), (48, 400, 1040)]


@pytest.fixture(scope="module")
def xp():
    import torch
    assert torch.cuda.is_available()
    from paper_2505_02146_amd import xp as m
    yield m
    for op in (0, 1, 2):
        for t in ("f32", "bf16", "i8"):
            m.xp_force_config(op, t, -1)


def _variants(xp, op, t):
    return list(range(xp.xp_num_configs(op, t))) + [-1]


def _make(kind, shape, seed, tid, integer=False):
    if kind == "i8":
        return inputs.int8_uniform(shape, seed, tid)
    x = inputs.small_integers(shape, seed, tid) if integer else inputs.normal(shape, seed, tid)
    return x if kind == "f32" else inputs.to_bf16_bits(x)


def _run_gemm(xp, oracle, kind, M, N, K, la, lb, lc="row", pads=(0, 0, 0), alpha=1.0, beta=0.0, integer=False,
              seed=1, variants=None):
    import torch
    A = _make(kind, (M, K), seed, 1, integer)
    B = _make(kind, (K, N), seed, 2, integer)
    a, lda = store(A, la, pads[0])
    b, ldb = store(B, lb, pads[1])
    out_np = np.int32 if kind == "i8" else np.float32
    C0 = inputs.small_integers((M, N), seed, 3).astype(out_np)
    c0, ldc = store(C0, lc, pads[2], fill=7)
    if kind == "i8":
        ref = oracle.gemm_i8(M, N, K, a, la, b, lb, lda=lda, ldb=ldb)
    else:
        ref = oracle.gemm_float(M, N, K, a, la, b, lb, lda=lda, ldb=ldb, alpha=alpha, beta=beta,
                                C0=c0 if beta != 0 else None, c_layout=lc, ldc=ldc)
    da, db = dev(a), dev(b)
    ran = 0
    for v in (variants if variants is not None else _variants(xp, 0, kind)):
        xp.xp_force_config(0, kind, v)
        if beta == 0 and kind != "i8":
            poison = c0.copy()
            poison[:] = np.nan                       # beta == 0 must not read C
            dc = dev(poison)
        else:
            dc = dev(c0)
        try:
            xp.xp_gemm(M, N, K, alpha, da, la, lda, db, lb, ldb, beta, dc, lc, ldc,
                       a_type=kind, b_type=kind)
        except xp.XpError as e:
            assert e.status == 6 and v > 0, (v, e)   # a forced tuned variant may decline a layout
            continue
        torch.cuda.synchronize()
        got_buf = dc.cpu().numpy()
        got = unstore(got_buf, lc, M, N, ldc)
        what = f"{kind} {M}x{N}x{K} {la}/{lb}/{lc} variant {v} ({xp.xp_last_config(0, kind)})"
        if kind == "i8" or integer:
            assert np.array_equal(got.astype(np.float64), ref.astype(np.float64)), what
        else:
            check_float(got, ref, what)
        # padding of C (between ld and the extent) must be untouched
        if pads[2]:
            full = got_buf.reshape(-1, ldc)
            ext = N if lc == "row" else M
            keep = c0.reshape(-1, ldc)[:, ext:] if beta != 0 or kind == "i8" else None
            if keep is not None:
                assert np.array_equal(full[:, ext:], keep), what + " wrote into the ld padding"
            else:
                assert np.all(np.isnan(full[:, ext:])), what + " wrote into the ld padding"
        ran += 1
    xp.xp_force_config(0, kind, -1)
    assert ran >= 2


@pytest.mark.parametrize("kind", ["f32", "bf16", "i8"])
@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_gemm_shapes_all_variants(xp, oracle, kind, la, lb):
    for (M, N, K) in SHAPES:
        _run_gemm(xp, oracle, kind, M, N, K, la, lb, seed=M + N)


@pytest.mark.parametrize("la,lb", [("row", "row"), ("col", "col"), ("col", "row")])
def test_gemm_operands_along_m_or_n_padding_alpha_beta(xp, oracle, la, lb):
    """The transposing-read kernels (operands contiguous along M / N) need extents that are multiples of 8:
    such shapes with padded leading dimensions, alpha and beta, several tiles, a ragged end of K, a K that is
    no multiple of 8 where no operand is K-contiguous, and a K long enough for the unrolled rounds."""
    names = [xp.xp_describe_config(0, "bf16", v) for v in range(xp.xp_num_configs(0, "bf16"))]
    outer = [v for v, n in enumerate(names) if "transposing reads" in n]
    assert len(outer) >= 6
    _run_gemm(xp, oracle, "bf16", 136, 72, 96, la, lb, lc="row", pads=(8, 16, 5), alpha=2.0, beta=3.0, integer=True, variants=outer + [-1])
    _run_gemm(xp, oracle, "bf16", 264, 520, 200, la, lb, lc="col", pads=(24, 8, 3), alpha=-0.5, beta=0.25, variants=outer + [-1])
    _run_gemm(xp, oracle, "bf16", 392, 136, 1544, la, lb, pads=(8, 8, 0), variants=outer + [-1])
    if (la, lb) == ("col", "row"):
        _run_gemm(xp, oracle, "bf16", 128, 256, 203, la, lb, variants=outer + [-1])


@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_gemm_integer_inputs_bit_exact(xp, oracle, kind):
    # every partial sum is an integer below 2^24: any summation order gives the same fp32 bits
    for (M, N, K) in [(64, 64, 64), (257, 130, 200), (300, 520, 1024)]:
        for la, lb in LAYOUTS[:2]:
            _run_gemm(xp, oracle, kind, M, N, K, la, lb, integer=True)


@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_gemm_alpha_beta_ld_padding_and_col_major_c(xp, oracle, kind):
    _run_gemm(xp, oracle, kind, 130, 70, 96, "row", "col", lc="row", pads=(8, 16, 5), alpha=2.0, beta=3.0, integer=True)
    _run_gemm(xp, oracle, kind, 130, 70, 96, "row", "col", lc="col", pads=(8, 8, 3), alpha=-0.5, beta=0.25)
    _run_gemm(xp, oracle, kind, 130, 70, 96, "col", "row", lc="col", pads=(8, 8, 2))
    _run_gemm(xp, oracle, kind, 70, 300, 40, "row", "col", lc="row", pads=(3, 5, 1))       # unaligned ld


@pytest.mark.parametrize("kind", ["bf16", "i8"])
def test_gemm_whole_tiles_with_alpha(xp, oracle, kind):
    """Tiles that lie inside the matrix take the epilogue's whole-tile path: with alpha != 1 (beta = 0), with alpha = 1,
    with a padded leading dimension of C, and with beta != 0 (which must fall back to the general path)."""
    _run_gemm(xp, oracle, kind, 512, 768, 136, "row", "col", alpha=1.0 if kind == "i8" else 0.75, beta=0.0, integer=True)   # (int8: no scaling)
    _run_gemm(xp, oracle, kind, 512, 512, 200, "row", "col", pads=(0, 0, 12), alpha=1.0, beta=0.0)
    # alpha = 1: the four-wave kernels store a block row behind the next one's MFMAs in the last K step -- that step as
    # the only one, as an even and as an odd one behind the unrolled rounds, with a partial step at the end
    for K in (64, 192, 512, 576, 1000):
        _run_gemm(xp, oracle, kind, 256, 512, K, "row", "col", alpha=1.0, beta=0.0, integer=(K == 512), seed=K)
    if kind != "i8":
        _run_gemm(xp, oracle, kind, 512, 512, 72, "row", "col", pads=(0, 0, 3), alpha=-1.5, beta=0.0)      # rows of C not 16-byte aligned
        _run_gemm(xp, oracle, kind, 512, 256, 72, "row", "col", alpha=0.5, beta=2.0, integer=True)


def test_gemm_int8_padding_and_col_major_c(xp, oracle):
    _run_gemm(xp, oracle, "i8", 130, 70, 96, "row", "col", lc="col", pads=(16, 32, 3))
    _run_gemm(xp, oracle, "i8", 70, 300, 40, "row", "col", lc="row", pads=(3, 5, 1))


def test_int8_extremes_on_gpu(xp, oracle):
    import torch
    M, N, K = 64, 64, 8192
    for va, vb, want in [(-128, -128, 2 ** 27), (-128, 127, -133169152)]:
        a = dev(np.full((M, K), va, np.int8))
        b = dev(np.full((N, K), vb, np.int8))
        for v in _variants(xp, 0, "i8"):
            xp.xp_force_config(0, "i8", v)
            c = torch.zeros((M, N), dtype=torch.int32, device="cuda")
            try:
                xp.xp_gemm(M, N, K, 1.0, a, "row", K, b, "col", K, 0.0, c, "row", N)
            except xp.XpError as e:
                assert e.status == 6 and v > 0       # a forced variant may decline this layout
                continue
            assert torch.all(c == want), (va, vb, v)
    xp.xp_force_config(0, "i8", -1)


def test_gemm_k_zero_and_closed_forms(xp, oracle):
    import torch
    # K == 0: C = beta * C
    c = torch.full((5, 7), 2.0, device="cuda")
    a = torch.zeros(1, device="cuda")
    xp.xp_gemm(5, 7, 0, 1.0, a, "row", 1, a, "row", 7, 3.0, c, "row", 7)
    assert torch.all(c == 6.0)
    c = torch.full((5, 7), float("nan"), device="cuda")
    xp.xp_gemm(5, 7, 0, 1.0, a, "row", 1, a, "row", 7, 0.0, c, "row", 7)
    assert torch.all(c == 0.0)
    # identity and all-ones through every bf16 variant
    n = 288
    eye = dev(inputs.to_bf16_bits(np.eye(n, dtype=np.float32)))
    x = inputs.to_bf16_bits(inputs.normal((n, n), 4, 1))
    dx = dev(x)
    ones = dev(inputs.to_bf16_bits(np.ones((n, n), np.float32)))
    for v in _variants(xp, 0, "bf16"):
        xp.xp_force_config(0, "bf16", v)
        c = torch.empty((n, n), device="cuda")
        try:
            xp.xp_gemm(n, n, n, 1.0, dx, "row", n, eye, "col", n, 0.0, c, "row", n, a_type="bf16", b_type="bf16")
        except xp.XpError as e:
            assert e.status == 6 and v > 0
            continue
        assert np.array_equal(c.cpu().numpy(), inputs.bf16_bits_to_f32(x)), v
        xp.xp_gemm(n, n, n, 1.0, ones, "row", n, ones, "col", n, 0.0, c, "row", n, a_type="bf16", b_type="bf16")
        assert torch.all(c == float(n)), v
    xp.xp_force_config(0, "bf16", -1)


@pytest.mark.parametrize("kind", ["f32", "bf16", "i8"])
def test_batched(xp, oracle, kind):
    import torch
    for batch, M, N, K, la, lb in [(1, 40, 50, 64, "row", "col"), (3, 129, 70, 80, "row", "col"),
                                   (3, 70, 64, 144, "row", "row"), (5, 33, 17, 16, "col", "col")]:
        sA, sB, sC = M * K + 16, K * N + 32, M * N + 8
        A = np.concatenate([np.concatenate([store(_make(kind, (M, K), 10 + i, 1), la)[0],
                                            np.zeros(16, _make(kind, (1, 1), 0, 1).dtype)]) for i in range(batch)])
        B = np.concatenate([np.concatenate([store(_make(kind, (K, N), 10 + i, 2), lb)[0],
                                            np.zeros(32, A.dtype)]) for i in range(batch)])
        lda = K if la == "row" else M
        ldb = N if lb == "row" else K
        if kind == "i8":
            ref = np.stack([oracle.gemm_i8(M, N, K, A[i * sA:i * sA + M * K].copy(), la,
                                           B[i * sB:i * sB + K * N].copy(), lb) for i in range(batch)])
        else:
            ref = oracle.gemm_float_batched(batch, M, N, K, A, la, B, lb, strideA=sA, strideB=sB)
        da, db = dev(A), dev(B)
        for v in _variants(xp, 1, kind):
            xp.xp_force_config(1, kind, v)
            c = torch.full((batch * sC,), 7, dtype=torch.int32 if kind == "i8" else torch.float32, device="cuda")
            try:
                xp.xp_gemm_batched(batch, M, N, K, 1.0, da, la, lda, sA, db, lb, ldb, sB, 0.0, c, "row", N, sC,
                                   a_type=kind, b_type=kind)
            except xp.XpError as e:
                assert e.status == 6 and v > 0
                continue
            got = c.cpu().numpy().reshape(batch, sC)
            assert np.all(got[:, M * N:] == 7), "wrote between the C slices"
            got = got[:, :M * N].reshape(batch, M, N)
            what = f"batched {kind} {batch}x{M}x{N}x{K} {la}/{lb} variant {v}"
            if kind == "i8":
                assert np.array_equal(got, ref), what
            else:
                check_float(got, ref, what)
        xp.xp_force_config(1, kind, -1)
    # shared B operand (strideB == 0)
    if kind != "i8":
        batch, M, N, K = 4, 64, 48, 32
        A = _make(kind, (batch, M, K), 3, 1)
        B = _make(kind, (N, K), 3, 2)
        ref = np.stack([oracle.gemm_float(M, N, K, A[i].reshape(-1), "row", B.reshape(-1), "col") for i in range(batch)])
        c = torch.empty((batch, M, N), device="cuda")
        xp.xp_gemm_batched(batch, M, N, K, 1.0, dev(A.reshape(-1)), "row", K, M * K, dev(B.reshape(-1)), "col", K, 0,
                           0.0, c, "row", N, M * N, a_type=kind, b_type=kind)
        check_float(c.cpu().numpy(), ref, "shared B")


CONV_CASES = [
    # N, H, W, Cin, Cout, R, S, stride, pad
    (2, 9, 7, 64, 40, 3, 3, (1, 1), (1, 1)),
    (1, 12, 12, 128, 96, 3, 3, (2, 2), (1, 1)),
    (2, 8, 10, 64, 64, 1, 1, (1, 1), (0, 0)),
    (1, 7, 9, 8, 5, 3, 2, (1, 2), (2, 1)),          # Cin not a multiple of the K step: general kernel
    (3, 6, 6, 192, 300, 2, 3, (1, 1), (0, 2)),
    (1, 20, 20, 64, 16, 5, 5, (3, 1), (2, 2)),
    # H = 1: one-dimensional convolutions (Table 5, "Conv1D") straight through the NHWC entry point
    (4, 1, 50, 64, 48, 1, 3, (1, 1), (0, 1)),
    (2, 1, 333, 128, 32, 1, 7, (1, 2), (0, 3)),
    (3, 1, 19, 5, 7, 1, 4, (1, 1), (0, 0)),          # few channels: general kernel
    # windows that stick out on both sides at once (image narrower than the filter), a tall one-column filter with
    # more padding than image rows at the stride, 32 taps (the whole padding mask): the MFMA kernels' mask arithmetic
    (2, 2, 3, 64, 32, 3, 5, (1, 1), (1, 2)),
    (1, 9, 4, 128, 16, 7, 1, (2, 1), (3, 0)),
    (1, 5, 11, 64, 24, 4, 8, (1, 3), (3, 7)),
]


@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("fl", ["krsc", "rsck"])
def test_conv_cases(xp, oracle, kind, fl):
    import torch
    for (N, H, W, Cin, Cout, R, S, stride, pad) in CONV_CASES:
        x = _make(kind, (N, H, W, Cin), 5, 1)
        w = _make(kind, (Cout, R, S, Cin), 5, 2)
        wbuf = w if fl == "krsc" else np.ascontiguousarray(w.transpose(1, 2, 3, 0))
        ref = oracle.conv2d_nhwc(x, wbuf, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S, stride=stride, pad=pad,
                                 filter_layout=fl)
        P, Q = ref.shape[1:3]
        dx, dw = dev(x.reshape(-1)), dev(wbuf.reshape(-1))
        ran = 0
        for v in _variants(xp, 2, kind):
            xp.xp_force_config(2, kind, v)
            out = torch.full((N, P, Q, Cout), float("nan"), device="cuda")
            try:
                xp.xp_conv2d_nhwc(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], dx, dw, fl, out,
                                  in_type=kind, w_type=kind)
            except xp.XpError as e:
                assert e.status == 6 and v > 0
                continue
            check_float(out.cpu().numpy(), ref, f"conv {kind} {fl} {(N, H, W, Cin, Cout, R, S, stride, pad)} variant {v}")
            ran += 1
        assert ran >= 2
    xp.xp_force_config(2, kind, -1)


def test_conv_closed_forms(xp):
    import torch
    # delta filter reproduces the input; shifted delta shifts it; all-ones counts valid taps
    N, H, W, C = 2, 10, 9, 64
    x = inputs.to_bf16_bits(inputs.normal((N, H, W, C), 2, 1))
    xf = inputs.bf16_bits_to_f32(x)
    w = np.zeros((C, 3, 3, C), np.float32)
    w[np.arange(C), 1, 1, np.arange(C)] = 1.0
    ws = np.zeros((C, 3, 3, C), np.float32)
    ws[np.arange(C), 0, 0, np.arange(C)] = 1.0
    ones_w = np.ones((C, 3, 3, C), np.float32)
    dx = dev(x.reshape(-1))
    for v in _variants(xp, 2, "bf16"):
        xp.xp_force_config(2, "bf16", v)
        out = torch.empty((N, H, W, C), device="cuda")
        try:
            xp.xp_conv2d_nhwc(N, H, W, C, C, 3, 3, 1, 1, 1, 1, dx, dev(inputs.to_bf16_bits(w).reshape(-1)), "krsc", out,
                              in_type="bf16", w_type="bf16")
        except xp.XpError as e:
            assert e.status == 6 and v > 0
            continue
        assert np.array_equal(out.cpu().numpy(), xf), v
        xp.xp_conv2d_nhwc(N, H, W, C, C, 3, 3, 1, 1, 1, 1, dx, dev(inputs.to_bf16_bits(ws).reshape(-1)), "krsc", out,
                          in_type="bf16", w_type="bf16")
        want = np.zeros_like(xf)
        want[:, 1:, 1:] = xf[:, :-1, :-1]
        assert np.array_equal(out.cpu().numpy(), want), v
        xp.xp_conv2d_nhwc(N, H, W, C, C, 3, 3, 1, 1, 1, 1, dev(inputs.to_bf16_bits(np.ones_like(xf)).reshape(-1)),
                          dev(inputs.to_bf16_bits(ones_w).reshape(-1)), "krsc", out, in_type="bf16", w_type="bf16")
        o = out.cpu().numpy()
        assert np.all(o[:, 1:-1, 1:-1] == 9 * C) and np.all(o[:, 0, 1:-1] == 6 * C) and np.all(o[:, 0, 0] == 4 * C), v
    xp.xp_force_config(2, "bf16", -1)


def test_stream_argument_is_used(xp, oracle):
    import torch
    M = N = K = 128
    A = inputs.uniform_pm1((M, K), 0, 1)
    B = inputs.uniform_pm1((K, N), 0, 2)
    ref = oracle.gemm_float(M, N, K, A.reshape(-1), "row", B.reshape(-1), "row")
    s = torch.cuda.Stream()
    da, db = dev(A), dev(B)
    c = torch.empty((M, N), device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        xp.xp_gemm(M, N, K, 1.0, da, "row", K, db, "row", N, 0.0, c, "row", N)
    s.synchronize()
    check_float(c.cpu().numpy(), ref, "side stream")


def _variant_named(xp, op, kind, fragment):
    for v in range(xp.xp_num_configs(op, kind)):
        if fragment in xp.xp_describe_config(op, kind, v):
            return v
    raise AssertionError(f"no variant named *{fragment}*")


def test_two_tile_heights_in_one_launch(xp, oracle):
    """Shapes whose rows spill over whole rounds of the tall tiles, so that both tile types of the
    two-height kernel run in the same launch (GEMM: 2 rounds of 224-row tiles + 208 rows of 192-row
    tiles with a ragged last tile; convolution: 1 round + 512 rows)."""
    import torch
    M, N, K = 2000, 16384, 136
    A = _make("bf16", (M, K), 9, 1)
    B = _make("bf16", (N, K), 9, 2)
    v = _variant_named(xp, 0, "bf16", "then 192x256 in the last round")
    xp.xp_force_config(0, "bf16", v)
    c = torch.full((M, N), float("nan"), device="cuda")
    xp.xp_gemm(M, N, K, 1.0, dev(A.reshape(-1)), "row", K, dev(B.reshape(-1)), "col", K, 0.0, c, "row", N,
               a_type="bf16", b_type="bf16")
    assert xp.xp_last_config(0, "bf16") == v
    xp.xp_force_config(0, "bf16", -1)
    check_float(c.cpu().numpy(), oracle.gemm_float(M, N, K, A.reshape(-1), "row", B.reshape(-1), "col"), "two heights gemm")

    n, h, w_, ci, co = 4, 32, 32, 64, 4096
    x = _make("bf16", (n, h, w_, ci), 9, 1)
    f = _make("bf16", (co, 3, 3, ci), 9, 2)
    v = _variant_named(xp, 2, "bf16", "then 192x256 in the last round")
    xp.xp_force_config(2, "bf16", v)
    out = torch.full((n, h, w_, co), float("nan"), device="cuda")
    xp.xp_conv2d_nhwc(n, h, w_, ci, co, 3, 3, 1, 1, 1, 1, dev(x.reshape(-1)), dev(f.reshape(-1)), "krsc", out,
                      in_type="bf16", w_type="bf16")
    assert xp.xp_last_config(2, "bf16") == v
    xp.xp_force_config(2, "bf16", -1)
    check_float(out.cpu().numpy(), oracle.conv2d_nhwc(x, f, N=n, H=h, W=w_, Cin=ci, Cout=co, R=3, S=3, pad=(1, 1)),
                "two heights conv")
