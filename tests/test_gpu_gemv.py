"""Matrix-vector products (GEMM with N == 1 or M == 1) on the GPU against the CPU oracle's GEMM,
through the C ABI, with the streaming kernel and with every other variant that accepts the call."""
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
    yield m
    for op in (0, 1):
        for t in ("f32", "bf16", "i8"):
            m.xp_force_config(op, t, -1)


def _gen(kind, shape, tid):
    if kind == "i8":
        return inputs.int8_uniform(shape, 5, tid)
    a = inputs.normal(shape, 5, tid).astype(np.float32)
    return inputs.to_bf16_bits(a) if kind == "bf16" else a


def _pad_rows(m, ld, fill):
    buf = np.full((m.shape[0], ld), fill, dtype=m.dtype)
    buf[:, :m.shape[1]] = m
    return buf.reshape(-1)


SHAPES = [(1, 8), (5, 24), (37, 104), (256, 4096), (1000, 72), (130, 1032), (4, 16384), (3, 40)]


@pytest.mark.parametrize("kind", ["f32", "bf16", "i8"])
@pytest.mark.parametrize("shape", SHAPES)
def test_matrix_times_vector(xp, oracle, kind, shape):
    import torch
    M, K = shape
    esz = {"f32": 4, "bf16": 2, "i8": 1}[kind]
    pad = ((K + 1) * esz + 15) // 16 * 16 // esz - K     # padded row pitch, a multiple of 16 bytes
    A, x = _gen(kind, (M, K), 1), _gen(kind, (1, K), 2)
    fill = {"f32": np.nan, "bf16": 0x7FC0, "i8": 77}[kind]
    Ab = _pad_rows(A, K + pad, fill)
    odt = torch.int32 if kind == "i8" else torch.float32
    xp.xp_force_config(0, kind, -1)
    ldc = 3                                         # the result vector need not be dense
    c = torch.full((M * ldc,), -7, dtype=odt, device="cuda")
    xp.xp_gemm(M, 1, K, 1.0, dev(Ab), "row", K + pad, dev(x.reshape(-1)), "col", K, 0.0, c, "row", ldc,
               a_type=kind, b_type=kind)
    assert "gemv" in xp.xp_describe_config(0, kind, xp.xp_last_config(0, kind))
    out = c.cpu().numpy().reshape(M, ldc)
    assert (out[:, 1:] == -7).all()
    if kind == "i8":
        ref = oracle.gemm_i8(M, 1, K, Ab, "row", x.reshape(-1), "col", lda=K + pad)
        assert np.array_equal(out[:, :1], ref)
    else:
        ref = oracle.gemm_float(M, 1, K, Ab, "row", x.reshape(-1), "col", lda=K + pad)
        check_float(out[:, :1], ref, f"gemv {kind} {shape}")


@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_alpha_beta(xp, oracle, kind):
    import torch
    M, K = 77, 200
    A, x = _gen(kind, (M, K), 1), _gen(kind, (1, K), 2)
    c0 = inputs.normal((M, 1), 5, 3).astype(np.float32)
    c = dev(c0.reshape(-1).copy())
    xp.xp_force_config(0, kind, -1)
    xp.xp_gemm(M, 1, K, 2.0, dev(A.reshape(-1)), "row", K, dev(x.reshape(-1)), "col", K, -3.0, c, "row", 1,
               a_type=kind, b_type=kind)
    assert "gemv" in xp.xp_describe_config(0, kind, xp.xp_last_config(0, kind))
    ref = oracle.gemm_float(M, 1, K, A.reshape(-1), "row", x.reshape(-1), "col", alpha=2.0, beta=-3.0, C0=c0.reshape(-1))
    check_float(c.cpu().numpy().reshape(M, 1), ref, "gemv alpha beta")


@pytest.mark.parametrize("kind", ["f32", "bf16", "i8"])
def test_row_vector_times_matrix(xp, oracle, kind):
    """M == 1: y = x.B with B stored column-major (its columns contiguous along K) is the same kernel."""
    import torch
    N, K = 300, 528
    x, Bt = _gen(kind, (1, K), 1), _gen(kind, (N, K), 2)        # Bt[n] is column n of B
    odt = torch.int32 if kind == "i8" else torch.float32
    c = torch.zeros((N,), dtype=odt, device="cuda")
    xp.xp_force_config(0, kind, -1)
    xp.xp_gemm(1, N, K, 1.0, dev(x.reshape(-1)), "row", K, dev(Bt.reshape(-1)), "col", K, 0.0, c, "row", N,
               a_type=kind, b_type=kind)
    assert "gemv" in xp.xp_describe_config(0, kind, xp.xp_last_config(0, kind))
    out = c.cpu().numpy().reshape(1, N)
    if kind == "i8":
        assert np.array_equal(out, oracle.gemm_i8(1, N, K, x.reshape(-1), "row", Bt.reshape(-1), "col"))
    else:
        check_float(out, oracle.gemm_float(1, N, K, x.reshape(-1), "row", Bt.reshape(-1), "col"), "row vector")
    # column-major 1 x N result: the dispatcher transposes twice and ends at the same kernel
    c2 = torch.zeros((N,), dtype=odt, device="cuda")
    xp.xp_gemm(1, N, K, 1.0, dev(x.reshape(-1)), "row", K, dev(Bt.reshape(-1)), "col", K, 0.0, c2, "col", 1,
               a_type=kind, b_type=kind)
    assert torch.equal(c, c2)


def test_batched_matrix_vector(xp, oracle):
    import torch
    b, M, K = 6, 50, 136
    A, x = _gen("bf16", (b, M, K), 1), _gen("bf16", (b, 1, K), 2)
    c = torch.full((b, M), float("nan"), device="cuda")
    xp.xp_force_config(1, "bf16", -1)
    xp.xp_gemm_batched(b, M, 1, K, 1.0, dev(A.reshape(-1)), "row", K, M * K, dev(x.reshape(-1)), "col", K, K, 0.0,
                       c, "row", 1, M, a_type="bf16", b_type="bf16")
    assert "gemv" in xp.xp_describe_config(1, "bf16", xp.xp_last_config(1, "bf16"))
    ref = oracle.gemm_float_batched(b, M, 1, K, A.reshape(-1), "row", x.reshape(-1), "col")
    check_float(c.cpu().numpy().reshape(b, M, 1), ref, "batched gemv")


def test_every_variant_that_accepts_a_vector_shape_agrees(xp, oracle):
    import torch
    M, K = 200, 264
    A, x = _gen("bf16", (M, K), 1), _gen("bf16", (1, K), 2)
    ref = oracle.gemm_float(M, 1, K, A.reshape(-1), "row", x.reshape(-1), "col")
    ran = 0
    for v in range(xp.xp_num_configs(0, "bf16")):
        xp.xp_force_config(0, "bf16", v)
        c = torch.full((M, 1), float("nan"), device="cuda")
        try:
            xp.xp_gemm(M, 1, K, 1.0, dev(A.reshape(-1)), "row", K, dev(x.reshape(-1)), "col", K, 0.0, c, "row", 1,
                       a_type="bf16", b_type="bf16")
        except xp.XpError as e:
            assert e.status == 6
            continue
        check_float(c.cpu().numpy(), ref, f"variant {v}")
        ran += 1
    assert ran >= 3


def test_layouts_the_streaming_kernel_declines_still_work(xp, oracle):
    import torch
    M, K = 90, 70
    A, x = _gen("f32", (K, M), 1), _gen("f32", (1, K), 2)       # A stored column-major: rows are not contiguous along K
    c = torch.full((M, 1), float("nan"), device="cuda")
    xp.xp_force_config(0, "f32", -1)
    xp.xp_gemm(M, 1, K, 1.0, dev(A.reshape(-1)), "col", M, dev(x.reshape(-1)), "col", K, 0.0, c, "row", 1)
    assert "gemv" not in xp.xp_describe_config(0, "f32", xp.xp_last_config(0, "f32"))
    check_float(c.cpu().numpy(), oracle.gemm_float(M, 1, K, A.reshape(-1), "col", x.reshape(-1), "col"), "col-major A")


def test_gemv_workload_full_size(xp, oracle):
    import torch
    w = inputs.workload("gemv_bf16_8192")
    M, K = w["M"], w["K"]
    c = torch.full((M, 1), float("nan"), device="cuda")
    xp.xp_force_config(0, "bf16", -1)
    xp.xp_gemm(M, 1, K, 1.0, dev(w["A"].reshape(-1)), "row", K, dev(w["B"].reshape(-1)), "col", K, 0.0, c, "row", 1,
               a_type="bf16", b_type="bf16")
    assert "gemv" in xp.xp_describe_config(0, "bf16", xp.xp_last_config(0, "bf16"))
    ref = oracle.gemm_float(M, 1, K, w["A"].reshape(-1), "row", w["B"].reshape(-1), "col")
    check_float(c.cpu().numpy(), ref, "gemv_bf16_8192")
