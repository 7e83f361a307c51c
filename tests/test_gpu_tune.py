"""The run-time parameter search (Section 5.1 of the paper, reward of Eq. 3-4) on the GPU: it picks a
valid variant, the library then uses it for that shape, the result still matches the CPU oracle, and
the table survives a save / clear / load cycle."""
import numpy as np
import pytest

from paper_2505_02146_amd import inputs
from tests.helpers import check_float, dev

pytestmark = pytest.mark.gpu


@pytest.fixture()
def xp():
    import torch
    assert torch.cuda.is_available()
    from paper_2505_02146_amd import xp as m
    for op in (0, 1, 2):
        for t in ("f32", "bf16", "i8"):
            m.xp_force_config(op, t, -1)
    m.xp_tune_clear()
    yield m
    m.xp_tune_clear()


def _ws(xp, extent):
    import torch
    return torch.empty(xp.xp_tune_workspace_bytes(extent), dtype=torch.uint8, device="cuda")


def test_tune_gemm_bf16_then_use_save_and_reload(xp, oracle, tmp_path):
    import torch
    M, N, K = 768, 640, 520
    A = inputs.to_bf16_bits(inputs.normal((M, K), 4, 1))
    B = inputs.to_bf16_bits(inputs.normal((N, K), 4, 2))
    dA, dB = dev(A.reshape(-1)), dev(B.reshape(-1))
    ref = oracle.gemm_float(M, N, K, A.reshape(-1), "row", B.reshape(-1), "col")

    def gemm(c):
        xp.xp_gemm(M, N, K, 1.0, dA, "row", K, dB, "col", K, 0.0, c, "row", N, a_type="bf16", b_type="bf16")

    c = torch.full((M, N), float("nan"), device="cuda")
    gemm(c)
    before = xp.xp_last_config(0, "bf16")
    c.fill_(float("nan"))
    best, us = xp.xp_tune_gemm(M, N, K, 1.0, dA, "row", K, dB, "col", K, 0.0, c, "row", N, _ws(xp, M * N), reps=10,
                               a_type="bf16", b_type="bf16")
    torch.cuda.synchronize()
    assert 0 < best < xp.xp_num_configs(0, "bf16") and us > 0        # some MFMA kernel beats the general one
    check_float(c.cpu().numpy(), ref, "C after tuning")               # the winner's result is left in C
    assert xp.xp_tune_count() == 1
    c.fill_(float("nan"))
    gemm(c)
    assert xp.xp_last_config(0, "bf16") == best                       # the library now uses the winner
    check_float(c.cpu().numpy(), ref, "tuned gemm")
    name = xp.xp_describe_config(0, "bf16", best)

    path = tmp_path / "tuned.txt"
    xp.xp_tune_save(path)
    assert name in path.read_text()
    xp.xp_tune_clear()
    gemm(c)
    assert xp.xp_last_config(0, "bf16") == before                     # back to the built-in choice
    xp.xp_tune_load(path)
    gemm(c)
    assert xp.xp_last_config(0, "bf16") == best
    # another shape is not affected
    c2 = torch.empty((64, 64), device="cuda")
    xp.xp_gemm(64, 64, 64, 1.0, dA, "row", K, dB, "col", K, 0.0, c2, "row", 64, a_type="bf16", b_type="bf16")
    assert xp.xp_tune_count() == 1
    # a forced variant still overrides the table
    xp.xp_force_config(0, "bf16", 0)
    gemm(c)
    assert xp.xp_last_config(0, "bf16") == 0
    xp.xp_force_config(0, "bf16", -1)


def test_tune_int8_is_bit_exact_and_beta_is_respected(xp, oracle):
    import torch
    M, N, K = 300, 272, 1040
    A, B = inputs.int8_uniform((M, K), 4, 1), inputs.int8_uniform((N, K), 4, 2)
    c = torch.zeros((M, N), dtype=torch.int32, device="cuda")
    best, us = xp.xp_tune_gemm(M, N, K, 1.0, dev(A.reshape(-1)), "row", K, dev(B.reshape(-1)), "col", K, 0.0, c, "row", N,
                               _ws(xp, M * N), reps=5)
    assert best >= 0 and us > 0
    assert np.array_equal(c.cpu().numpy(), oracle.gemm_i8(M, N, K, A.reshape(-1), "row", B.reshape(-1), "col"))

    # fp32 with alpha, beta and a padded, column-major C: the input C must survive the candidates
    M, N, K = 130, 70, 90
    Af, Bf = inputs.normal((M, K), 4, 1).astype(np.float32), inputs.normal((K, N), 4, 2).astype(np.float32)
    ldc = M + 5
    c0 = inputs.normal((N, ldc), 4, 3).astype(np.float32)
    cf = dev(c0.reshape(-1).copy())
    best, us = xp.xp_tune_gemm(M, N, K, 1.5, dev(Af.reshape(-1)), "row", K, dev(Bf.reshape(-1)), "row", N, -0.5, cf, "col", ldc,
                               _ws(xp, (N - 1) * ldc + M), reps=5)
    ref = oracle.gemm_float(M, N, K, Af.reshape(-1), "row", Bf.reshape(-1), "row", alpha=1.5, beta=-0.5,
                            C0=c0.reshape(-1), c_layout="col", ldc=ldc)
    got = cf.cpu().numpy().reshape(N, ldc)
    check_float(got[:, :M].T, ref, "tuned fp32 alpha/beta col-major")
    assert np.array_equal(got[:, M:], c0[:, M:])                      # padding untouched


def test_tune_batched_and_conv(xp, oracle):
    import torch
    b, M, N, K = 6, 256, 192, 64
    A = inputs.to_bf16_bits(inputs.normal((b, M, K), 4, 1))
    B = inputs.to_bf16_bits(inputs.normal((b, N, K), 4, 2))
    c = torch.full((b, M, N), float("nan"), device="cuda")
    best, us = xp.xp_tune_gemm_batched(b, M, N, K, 1.0, dev(A.reshape(-1)), "row", K, M * K, dev(B.reshape(-1)), "col", K,
                                       N * K, 0.0, c, "row", N, M * N, _ws(xp, b * M * N), reps=5,
                                       a_type="bf16", b_type="bf16")
    assert best > 0
    check_float(c.cpu().numpy(), oracle.gemm_float_batched(b, M, N, K, A.reshape(-1), "row", B.reshape(-1), "col"), "batched")

    n, h, w_, ci, co = 2, 20, 20, 64, 128
    x = inputs.to_bf16_bits(inputs.normal((n, h, w_, ci), 4, 1))
    f = inputs.to_bf16_bits(inputs.normal((co, 3, 3, ci), 4, 2, 1.0 / 24.0))
    out = torch.full((n, h, w_, co), float("nan"), device="cuda")
    dx, df = dev(x.reshape(-1)), dev(f.reshape(-1))
    best, us = xp.xp_tune_conv2d_nhwc(n, h, w_, ci, co, 3, 3, 1, 1, 1, 1, dx, df, "krsc", out, _ws(xp, n * h * w_ * co),
                                      reps=5, in_type="bf16", w_type="bf16")
    assert best > 0
    ref = oracle.conv2d_nhwc(x, f, N=n, H=h, W=w_, Cin=ci, Cout=co, R=3, S=3, pad=(1, 1))
    check_float(out.cpu().numpy(), ref, "tuned conv")
    out.fill_(float("nan"))
    xp.xp_conv2d_nhwc(n, h, w_, ci, co, 3, 3, 1, 1, 1, 1, dx, df, "krsc", out, in_type="bf16", w_type="bf16")
    assert xp.xp_last_config(2, "bf16") == best
    check_float(out.cpu().numpy(), ref, "conv with the tuned variant")
    assert xp.xp_tune_count() == 2


def test_workspace_too_small_is_refused(xp):
    import torch
    a = torch.zeros(64 * 64, dtype=torch.int16, device="cuda")
    c = torch.zeros((64, 64), device="cuda")
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(xp.XpError) as e:
        xp.xp_tune_gemm(64, 64, 64, 1.0, a, "row", 64, a, "col", 64, 0.0, c, "row", 64, small, reps=3, a_type="bf16",
                        b_type="bf16")
    assert e.value.status == 8
    assert xp.xp_tune_count() == 0


def test_two_convolutions_with_equal_gemm_extents_keep_their_own_winners(xp, tmp_path):
    """A 3x3 convolution over 64 channels and a 1x1 convolution over 576 have the same implicit-GEMM extents
    (M = N*P*Q, N = Cout, K = R*S*Cin).  The table of tuned shapes tells them apart by geometry, and so must the
    per-thread memory of recent selections: each call gets the variant recorded for its own geometry, in any order."""
    import torch
    N, H, W, Cout = 2, 16, 16, 64
    geo_a = (N, H, W, 64, Cout, 3, 3, 1, 1, 1, 1)
    geo_b = (N, H, W, 576, Cout, 1, 1, 1, 1, 0, 0)
    xa, wa = (torch.randn(N, H, W, 64, device="cuda").bfloat16(), (torch.randn(Cout, 3, 3, 64, device="cuda") / 24).bfloat16())
    xb, wb = (torch.randn(N, H, W, 576, device="cuda").bfloat16(), (torch.randn(Cout, 1, 1, 576, device="cuda") / 24).bfloat16())
    out = torch.empty(N, H, W, Cout, device="cuda")

    def call(geo, x, w):
        xp.xp_conv2d_nhwc(*geo, x, w, "krsc", out)
        return xp.xp_last_config(2, "bf16")

    # record both shapes once (whatever wins), to obtain the table's own spelling of the two keys
    ws = _ws(xp, N * H * W * Cout)
    xp.xp_tune_conv2d_nhwc(*geo_a, xa, wa, "krsc", out, ws, reps=3)
    xp.xp_tune_conv2d_nhwc(*geo_b, xb, wb, "krsc", out, ws, reps=3)
    path = tmp_path / "two.txt"
    xp.xp_tune_save(path)
    lines = [l for l in path.read_text().splitlines() if " | " in l and not l.startswith("#")]
    assert len(lines) == 2
    key_a = next(l for l in lines if " c64 " in l).split(" | ")[0]
    key_b = next(l for l in lines if " c576 " in l).split(" | ")[0]
    # two different variants that can run both calls: the general kernel and the first register-staged MFMA kernel
    name_x = xp.xp_describe_config(2, "bf16", 0)
    idx_y = next(i for i in range(1, xp.xp_num_configs(2, "bf16")) if "direct-to-lds" not in xp.xp_describe_config(2, "bf16", i)
                 and "mfma" in xp.xp_describe_config(2, "bf16", i))
    name_y = xp.xp_describe_config(2, "bf16", idx_y)
    path.write_text(f"{key_a} | {name_x}\n{key_b} | {name_y}\n")
    xp.xp_tune_clear()
    xp.xp_tune_load(path)
    assert call(geo_a, xa, wa) == 0
    assert call(geo_b, xb, wb) == idx_y
    assert call(geo_a, xa, wa) == 0
    assert call(geo_b, xb, wb) == idx_y
