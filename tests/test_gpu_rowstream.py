"""The row-streaming kernel (few columns, short reduction, row-major B: the P.V stage of an attention block) forced
through the C ABI against the CPU oracle: ragged row counts, N and K below their maxima, padded pitches,
alpha / beta, exact integer data, a strided batch with gaps, and the workload's own shape."""
import numpy as np
import pytest

from paper_2505_02146_amd import inputs
from tests.helpers import check_float, dev, store, unstore

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xp():
    import torch
    assert torch.cuda.is_available()
    from paper_2505_02146_amd import xp as m
    yield m
    for op in (0, 1):
        m.xp_force_config(op, "bf16", -1)


def _variant(xp, op):
    names = [xp.xp_describe_config(op, "bf16", v) for v in range(xp.xp_num_configs(op, "bf16"))]
    hits = [v for v, n in enumerate(names) if "row-streaming" in n]
    assert len(hits) == 1, names
    return hits[0]


CASES = [  # M, N, K, pads (lda, ldb, ldc), alpha, beta, integer data
    (300, 64, 512, (0, 0, 0), 1.0, 0.0, False),
    (1000, 40, 264, (8, 24, 5), 2.0, 3.0, True),          # N and K below the maxima, padded pitches, beta reads C
    (77, 8, 8, (0, 8, 0), 1.0, 0.0, False),               # one chunk of K and of N, a ragged last block row
    (64, 64, 256, (0, 0, 0), -0.5, 0.25, False),          # a single half of K
    (513, 56, 320, (16, 8, 3), 1.0, 0.0, True),           # second half of K partly filled
    (16, 64, 512, (0, 0, 0), 1.0, 0.0, False),            # one block row: three waves of the workgroup have nothing to do
    (4099, 64, 512, (0, 0, 0), 1.0, 0.0, False),          # many workgroups, the last one ragged
]


@pytest.mark.parametrize("case", CASES)
def test_rowstream_gemm(xp, oracle, case):
    import torch
    M, N, K, pads, alpha, beta, integer = case
    v = _variant(xp, 0)
    A = inputs.small_integers((M, K), M, 1) if integer else inputs.normal((M, K), M, 1)
    B = inputs.small_integers((K, N), M, 2) if integer else inputs.normal((K, N), M, 2)
    a, lda = store(inputs.to_bf16_bits(A), "row", pads[0])
    b, ldb = store(inputs.to_bf16_bits(B), "row", pads[1])
    C0 = inputs.small_integers((M, N), M, 3).astype(np.float32)
    c0, ldc = store(C0, "row", pads[2], fill=7)
    ref = oracle.gemm_float(M, N, K, a, "row", b, "row", lda=lda, ldb=ldb, alpha=alpha, beta=beta,
                            C0=c0 if beta != 0 else None, c_layout="row", ldc=ldc)
    start = c0.copy()
    if beta == 0:
        start[:] = np.nan                                 # beta == 0 must not read C
    dc = dev(start)
    xp.xp_force_config(0, "bf16", v)
    try:
        xp.xp_gemm(M, N, K, alpha, dev(a), "row", lda, dev(b), "row", ldb, beta, dc, "row", ldc, a_type="bf16", b_type="bf16")
    finally:
        xp.xp_force_config(0, "bf16", -1)
    torch.cuda.synchronize()
    assert xp.xp_last_config(0, "bf16") == v
    buf = dc.cpu().numpy()
    got = unstore(buf, "row", M, N, ldc)
    if integer:
        assert np.array_equal(got.astype(np.float64), ref), case
    else:
        check_float(got, ref, f"row-streaming {case}")
    if pads[2]:
        tail = buf.reshape(-1, ldc)[:, N:]
        assert np.all(np.isnan(tail)) if beta == 0 else np.array_equal(tail, c0.reshape(-1, ldc)[:, N:]), "wrote into the ld padding"


def test_rowstream_declines_what_it_cannot_hold(xp):
    import torch
    v = _variant(xp, 0)
    a = torch.zeros(64 * 1024, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(64 * 128, device="cuda")
    xp.xp_force_config(0, "bf16", v)
    try:
        for (M, N, K, lb) in [(64, 128, 64, "row"), (64, 64, 1024, "row"), (64, 64, 64, "col"), (64, 60, 64, "row")]:
            with pytest.raises(xp.XpError) as e:
                xp.xp_gemm(M, N, K, 1.0, a, "row", K, a, lb, N if lb == "row" else K, 0.0, c, "row", N)
            assert e.value.status == 6
    finally:
        xp.xp_force_config(0, "bf16", -1)


def test_rowstream_batched_with_gaps_and_workload(xp, oracle):
    import torch
    v = _variant(xp, 1)
    # a small batch with gaps between the problems of every operand
    batch, M, N, K = 5, 130, 48, 200
    sA, sB, sC = M * K + 64, K * N + 8, M * N + 12
    A = inputs.to_bf16_bits(inputs.normal((batch, M, K), 3, 1))
    B = inputs.to_bf16_bits(inputs.normal((batch, K, N), 3, 2))
    a = np.zeros(batch * sA, np.uint16); b = np.zeros(batch * sB, np.uint16)
    for i in range(batch):
        a[i * sA:i * sA + M * K] = A[i].reshape(-1)
        b[i * sB:i * sB + K * N] = B[i].reshape(-1)
    ref = oracle.gemm_float_batched(batch, M, N, K, a, "row", b, "row", strideA=sA, strideB=sB)
    dc = torch.full((batch * sC,), 7.0, device="cuda")
    xp.xp_force_config(1, "bf16", v)
    try:
        xp.xp_gemm_batched(batch, M, N, K, 1.0, dev(a), "row", K, sA, dev(b), "row", N, sB, 0.0, dc, "row", N, sC,
                           a_type="bf16", b_type="bf16")
        got = dc.cpu().numpy().reshape(batch, sC)
        assert np.all(got[:, M * N:] == 7), "wrote between the C slices"
        check_float(got[:, :M * N].reshape(batch, M, N), ref, "row-streaming batched with gaps")
        # the workload: 96 x (512 x 64 x 512)
        w = inputs.workload("bgemm_bf16_pv")
        bb, m, n, k = w["batch"], w["M"], w["N"], w["K"]
        c = torch.full((bb, m, n), float("nan"), device="cuda")
        xp.xp_gemm_batched(bb, m, n, k, 1.0, dev(w["A"].reshape(-1)), "row", k, m * k, dev(w["B"].reshape(-1)), "row", n, k * n,
                           0.0, c, "row", n, m * n, a_type="bf16", b_type="bf16")
        assert xp.xp_last_config(1, "bf16") == v
        check_float(c.cpu().numpy(), oracle.gemm_float_batched(bb, m, n, k, w["A"].reshape(-1), "row", w["B"].reshape(-1), "row"),
                    "row-streaming on the P.V workload")
    finally:
        xp.xp_force_config(1, "bf16", -1)
