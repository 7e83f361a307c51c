"""The five benchmark workloads at full size, in the launch configuration the benchmark times
(the library's own variant selection), checked against the CPU oracle over the WHOLE output (the
oracle finishes each of them in seconds on the host cores), with row/column checksums that follow from
linearity as a second line of defence:  1^T C = (1^T A) B  and  C 1 = A (B 1)  (fp64, numpy).
The same product in the other operand layouts is checked on sampled full rows and columns."""
import numpy as np
import pytest

from paper_2505_02146_amd import inputs
from tests.helpers import check_float, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xp():
    import torch
    assert torch.cuda.is_available()
    from paper_2505_02146_amd import xp as m
    for op in (0, 1, 2):
        for t in ("f32", "bf16", "i8"):
            m.xp_force_config(op, t, -1)
    return m


def _f64(x):
    return inputs.bf16_bits_to_f32(x).astype(np.float64) if x.dtype == np.uint16 else x.astype(np.float64)


def test_gemm_f32_256(xp, oracle):
    import torch
    w = inputs.workload("gemm_f32_256")
    M, N, K = w["M"], w["N"], w["K"]
    c = torch.full((M, N), float("nan"), device="cuda")
    xp.xp_gemm(M, N, K, 1.0, dev(w["A"]), "row", K, dev(w["B"]), "row", N, 0.0, c, "row", N)
    ref = oracle.gemm_float(M, N, K, w["A"].reshape(-1), "row", w["B"].reshape(-1), "row")
    check_float(c.cpu().numpy(), ref, "gemm_f32_256")
    assert xp.xp_last_config(0, "f32") > 0, "the MFMA kernel, not the general one, must serve this workload"


def _checksums(w, kind, got):
    """Whole-output checksums from linearity (independent of the oracle library)."""
    M, K = w["M"], w["K"]
    A, B = w["A"], w["B"]                       # A: M x K row-major, B: N x K (column-major K x N)
    if kind == "i8":                            # exact in int64
        assert np.array_equal(got.astype(np.int64).sum(0), A.astype(np.int64).sum(0) @ B.astype(np.int64).T)
        assert np.array_equal(got.astype(np.int64).sum(1), A.astype(np.int64) @ B.astype(np.int64).sum(0))
    else:
        Af, Bf = _f64(A), _f64(B)
        scale = np.sqrt(M * K) * float(np.sqrt(np.mean(Af[:64] ** 2) * np.mean(Bf[:64] ** 2)))
        g = got.astype(np.float64)
        assert np.max(np.abs(g.sum(0) - Af.sum(0) @ Bf.T)) <= 1e-3 * scale
        assert np.max(np.abs(g.sum(1) - Af @ Bf.sum(0))) <= 1e-3 * scale


def _full_gemm_check(oracle, w, kind, got, what):
    """Every element of the output against the oracle."""
    M, N, K = w["M"], w["N"], w["K"]
    if kind == "i8":
        ref = oracle.gemm_i8(M, N, K, w["A"].reshape(-1), "row", w["B"].reshape(-1), "col")
        assert np.array_equal(got, ref), f"{what}: {int(np.count_nonzero(got != ref))} of {ref.size} elements differ"
    else:
        ref = oracle.gemm_float(M, N, K, w["A"].reshape(-1), "row", w["B"].reshape(-1), "col")
        check_float(got, ref, what)
    _checksums(w, kind, got)


def _sampled_gemm_check(xp, oracle, w, kind, got, rng):
    M, N, K = w["M"], w["N"], w["K"]
    A, B = w["A"], w["B"]
    rows = np.sort(rng.choice(M, 48, replace=False))
    cols = np.sort(rng.choice(N, 48, replace=False))
    rows[0], rows[-1], cols[0], cols[-1] = 0, M - 1, 0, N - 1
    ref_r = oracle.gemm_float(len(rows), N, K, np.ascontiguousarray(A[rows]).reshape(-1), "row", B.reshape(-1), "col")
    ref_c = oracle.gemm_float(M, len(cols), K, A.reshape(-1), "row", np.ascontiguousarray(B[cols]).reshape(-1), "col")
    check_float(got[rows], ref_r, "sampled rows")
    check_float(got[:, cols], ref_c, "sampled columns")
    _checksums(w, kind, got)


def test_gemm_bf16_4096(xp, oracle):
    import torch
    w = inputs.workload("gemm_bf16_4096")
    M, N, K = w["M"], w["N"], w["K"]
    c = torch.full((M, N), float("nan"), device="cuda")
    xp.xp_gemm(M, N, K, 1.0, dev(w["A"].reshape(-1)), "row", K, dev(w["B"].reshape(-1)), "col", K, 0.0, c, "row", N,
               a_type="bf16", b_type="bf16")
    assert xp.xp_last_config(0, "bf16") > 0
    _full_gemm_check(oracle, w, "bf16", c.cpu().numpy(), "gemm_bf16_4096, all 4096 x 4096 elements")


@pytest.mark.parametrize("la,lb", [("row", "row"), ("col", "col"), ("col", "row")])
def test_gemm_bf16_4096_other_layouts(xp, oracle, la, lb):
    """The same 4096^3 product with its operands stored the other way round (row-major B, column-major A, both):
    the library's own selection -- the transposing-read kernels -- against the same sampled rows, columns
    and checksums."""
    import torch
    w = inputs.workload("gemm_bf16_4096")
    M, N, K = w["M"], w["N"], w["K"]
    A, B = w["A"], w["B"]                       # A: M x K, B: N x K
    a = A if la == "row" else np.ascontiguousarray(A.T)     # col: stored K x M
    b = B if lb == "col" else np.ascontiguousarray(B.T)     # row: stored K x N
    c = torch.full((M, N), float("nan"), device="cuda")
    xp.xp_gemm(M, N, K, 1.0, dev(a.reshape(-1)), la, K if la == "row" else M, dev(b.reshape(-1)), lb, K if lb == "col" else N,
               0.0, c, "row", N, a_type="bf16", b_type="bf16")
    name = xp.xp_describe_config(0, "bf16", xp.xp_last_config(0, "bf16"))
    assert "transposing reads" in name, name
    _sampled_gemm_check(xp, oracle, w, "bf16", c.cpu().numpy(), np.random.default_rng(1))


def test_gemm_i8_4096x4096x8192(xp, oracle):
    import torch
    w = inputs.workload("gemm_i8_4096x4096x8192")
    M, N, K = w["M"], w["N"], w["K"]
    c = torch.full((M, N), -1, dtype=torch.int32, device="cuda")
    xp.xp_gemm(M, N, K, 1.0, dev(w["A"].reshape(-1)), "row", K, dev(w["B"].reshape(-1)), "col", K, 0.0, c, "row", N)
    assert xp.xp_last_config(0, "i8") > 0
    _full_gemm_check(oracle, w, "i8", c.cpu().numpy(), "gemm_i8_4096x4096x8192, all 4096 x 4096 elements")


@pytest.mark.parametrize("name", ["bgemm_bf16_qk", "bgemm_bf16_pv"])
def test_batched_attention_shapes(xp, oracle, name):
    import torch
    w = inputs.workload(name)
    b, M, N, K = w["batch"], w["M"], w["N"], w["K"]
    lb = w["b_layout"]
    ldb = N if lb == "row" else K
    c = torch.full((b, M, N), float("nan"), device="cuda")
    xp.xp_gemm_batched(b, M, N, K, 1.0, dev(w["A"].reshape(-1)), "row", K, M * K, dev(w["B"].reshape(-1)), lb, ldb,
                       K * N, 0.0, c, "row", N, M * N, a_type="bf16", b_type="bf16")
    got = c.cpu().numpy()
    # the whole batch is 3.2 GFLOP: the oracle does all of it
    ref = oracle.gemm_float_batched(b, M, N, K, w["A"].reshape(-1), "row", w["B"].reshape(-1), lb)
    check_float(got, ref, name)


def test_conv_bf16_56(xp, oracle):
    import torch
    w = inputs.workload("conv_bf16_56")
    N, H, W, Cin, Cout, R, S = (w[k] for k in ("N", "H", "W", "Cin", "Cout", "R", "S"))
    out = torch.full((N, H, W, Cout), float("nan"), device="cuda")
    xp.xp_conv2d_nhwc(N, H, W, Cin, Cout, R, S, 1, 1, 1, 1, dev(w["input"].reshape(-1)), dev(w["filter"].reshape(-1)),
                      "krsc", out, in_type="bf16", w_type="bf16")
    assert xp.xp_last_config(2, "bf16") > 0
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    # all 32 images through the oracle (a few seconds on the host cores)
    ref = oracle.conv2d_nhwc(w["input"], w["filter"], N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S, pad=(1, 1))
    check_float(got, ref, "conv_bf16_56, all 32 images")
    for n in (0, 13, N - 1):                     # and image by image, so that a failure names the image
        check_float(got[n:n + 1], ref[n:n + 1], f"conv image {n}")
    # whole-output checksum: summing the output over channels k equals convolving with the
    # channel-summed filter; evaluated per image as sum over all positions (fp64, numpy)
    x = _f64(w["input"])
    f = _f64(w["filter"])                        # K R S C
    fsum = f.sum(0)                              # R S C
    xp_ = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    want = np.zeros(N)
    for r in range(R):
        for s in range(S):
            want += np.einsum("nhwc,c->n", xp_[:, r:r + H, s:s + W], fsum[r, s])
    total = got.astype(np.float64).sum(axis=(1, 2, 3))
    assert np.max(np.abs(total - want)) <= 1e-3 * np.sqrt(H * W * Cout * R * S * Cin) * 1.0 / 48.0


def test_repeated_launches_give_the_same_bits(xp):
    """Every kernel here sums a fixed order, so a launch repeated on the same inputs must reproduce its output bit
    for bit; a mismatch would mean that a wave read an LDS buffer before its loads had landed or after it was refilled.
    The MFMA-bound workloads, 40 launches each in the library's own selection, while other launches keep the chip busy."""
    import torch
    w = inputs.workload("gemm_bf16_4096")
    M, N, K = w["M"], w["N"], w["K"]
    a, b = dev(w["A"].reshape(-1)), dev(w["B"].reshape(-1))
    wi = inputs.workload("gemm_i8_4096x4096x8192")
    Mi, Ni, Ki = wi["M"], wi["N"], wi["K"]
    ai, bi = dev(wi["A"].reshape(-1)), dev(wi["B"].reshape(-1))
    wc = inputs.workload("conv_bf16_56")
    xin, fil = dev(wc["input"].reshape(-1)), dev(wc["filter"].reshape(-1))
    c = [torch.empty((M, N), device="cuda") for _ in range(2)]
    ci = [torch.empty((Mi, Ni), dtype=torch.int32, device="cuda") for _ in range(2)]
    cc = [torch.empty((32, 56, 56, 256), device="cuda") for _ in range(2)]
    for it in range(40):
        k = min(it, 1)
        xp.xp_gemm(M, N, K, 1.0, a, "row", K, b, "col", K, 0.0, c[k], "row", N, a_type="bf16", b_type="bf16")
        xp.xp_gemm(Mi, Ni, Ki, 1.0, ai, "row", Ki, bi, "col", Ki, 0.0, ci[k], "row", Ni, a_type="i8", b_type="i8")
        xp.xp_conv2d_nhwc(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, xin, fil, "krsc", cc[k], in_type="bf16", w_type="bf16")
        if it >= 1:
            assert torch.equal(c[0].view(torch.int32), c[1].view(torch.int32)), f"bf16 GEMM, launch {it}"
            assert torch.equal(ci[0], ci[1]), f"int8 GEMM, launch {it}"
            assert torch.equal(cc[0].view(torch.int32), cc[1].view(torch.int32)), f"convolution, launch {it}"
