"""NCHW convolution on the GPU (layout change + the NHWC kernels) against the CPU oracle's NCHW loop."""
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
    m.xp_force_config(2, "bf16", -1)
    m.xp_force_config(2, "f32", -1)
    return m


CASES = [  # N, H, W, Cin, Cout, R, S, stride, pad
    (2, 9, 11, 64, 96, 3, 3, (1, 1), (1, 1)),
    (1, 7, 5, 3, 8, 3, 2, (2, 1), (1, 2)),               # few channels: the general kernel underneath
    (3, 14, 14, 128, 70, 1, 1, (1, 1), (0, 0)),
    (1, 16, 16, 64, 64, 5, 5, (2, 2), (2, 2)),
    (2, 1, 40, 64, 32, 1, 3, (1, 1), (0, 1)),            # H = 1: a 1-D convolution
]


@pytest.mark.parametrize("kind", ["bf16", "f32"])
def test_conv_nchw_cases(xp, oracle, kind):
    import torch
    for (N, H, W, Cin, Cout, R, S, stride, pad) in CASES:
        x = inputs.normal((N, Cin, H, W), 8, 1).astype(np.float32)
        w = inputs.normal((Cout, Cin, R, S), 8, 2, 1.0 / np.sqrt(R * S * Cin)).astype(np.float32)
        if kind == "bf16":
            x, w = inputs.to_bf16_bits(x), inputs.to_bf16_bits(w)
        ref = oracle.conv2d_nchw(x, w, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S, stride=stride, pad=pad)
        need = xp.xp_conv2d_nchw_workspace_bytes(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], kind)
        assert need > 0
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        out = torch.full(ref.shape, float("nan"), device="cuda")
        xp.xp_conv2d_nchw(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], dev(x.reshape(-1)), dev(w.reshape(-1)),
                          out, ws, in_type=kind, w_type=kind)
        check_float(out.cpu().numpy(), ref, f"conv nchw {kind} {(N, H, W, Cin, Cout, R, S, stride, pad)}")
        small = torch.empty(need - 1, dtype=torch.uint8, device="cuda")
        with pytest.raises(xp.XpError) as e:
            xp.xp_conv2d_nchw(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], dev(x.reshape(-1)),
                              dev(w.reshape(-1)), out, small, in_type=kind, w_type=kind)
        assert e.value.status == 8


def test_conv_nchw_resnet_stage_sampled(xp, oracle):
    """The convolution workload's shape in NCHW: 8 images checked in full against the oracle."""
    import torch
    N, H, W, C = 32, 56, 56, 256
    x = inputs.to_bf16_bits(inputs.normal((N, C, H, W), 0, 1))
    w = inputs.to_bf16_bits(inputs.normal((C, C, 3, 3), 0, 2, 1.0 / 48.0))
    ws = torch.empty(xp.xp_conv2d_nchw_workspace_bytes(N, H, W, C, C, 3, 3, 1, 1, 1, 1, "bf16"), dtype=torch.uint8, device="cuda")
    out = torch.full((N, C, H, W), float("nan"), device="cuda")
    xp.xp_conv2d_nchw(N, H, W, C, C, 3, 3, 1, 1, 1, 1, dev(x.reshape(-1)), dev(w.reshape(-1)), out, ws, in_type="bf16", w_type="bf16")
    got = out.cpu().numpy()
    for n in (0, 31):
        ref = oracle.conv2d_nchw(np.ascontiguousarray(x[n:n + 1]), w, N=1, H=H, W=W, Cin=C, Cout=C, R=3, S=3, pad=(1, 1))
        check_float(got[n:n + 1], ref, f"nchw workload image {n}")


def test_every_variant_writes_planes_or_declines(xp, oracle):
    """Forced through each convolution variant: it either declines the planar output or produces it."""
    import torch
    N, H, W, Cin, Cout = 3, 13, 10, 64, 80                     # P*Q = 130: 16-row blocks straddle the images
    x = inputs.to_bf16_bits(inputs.normal((N, Cin, H, W), 9, 1))
    w = inputs.to_bf16_bits(inputs.normal((Cout, Cin, 3, 3), 9, 2, 1.0 / 24.0))
    ref = oracle.conv2d_nchw(x, w, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=3, S=3, pad=(1, 1))
    ws = torch.empty(xp.xp_conv2d_nchw_workspace_bytes(N, H, W, Cin, Cout, 3, 3, 1, 1, 1, 1, "bf16"), dtype=torch.uint8, device="cuda")
    ran = []
    try:
        for idx in range(xp.xp_num_configs(2, "bf16")):
            xp.xp_force_config(2, "bf16", idx)
            out = torch.full(ref.shape, float("nan"), device="cuda")
            try:
                xp.xp_conv2d_nchw(N, H, W, Cin, Cout, 3, 3, 1, 1, 1, 1, dev(x.reshape(-1)), dev(w.reshape(-1)), out, ws,
                                  in_type="bf16", w_type="bf16")
            except xp.XpError as e:
                assert e.status == 6, (idx, e.status)                  # XP_ERR_CONFIG: this variant cannot run the call
                continue
            check_float(out.cpu().numpy(), ref, f"planar output, variant {idx}: {xp.xp_describe_config(2, 'bf16', idx)}")
            ran.append(idx)
    finally:
        xp.xp_force_config(2, "bf16", -1)
    assert 0 in ran and len(ran) >= 5, ran                     # the general kernel and the 16x16-block direct-to-LDS kernels
