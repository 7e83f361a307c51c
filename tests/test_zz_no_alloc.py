"""xp_conv2d_nchw_static (the entry point that allocates nothing) against xp_conv2d_nchw, through the C ABI."""
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


def _both(xp, oracle, kind, N, H, W, Cin, Cout, R, S, stride, pad, seed):
    """Runs the workspace entry point and the static one on the same inputs; returns both outputs."""
    import torch
    x = inputs.normal((N, Cin, H, W), seed, 1).astype(np.float32)
    w = inputs.normal((Cout, Cin, R, S), seed, 2, 1.0 / np.sqrt(R * S * Cin)).astype(np.float32)
    if kind == "bf16":
        x, w = inputs.to_bf16_bits(x), inputs.to_bf16_bits(w)
    need = xp.xp_conv2d_nchw_workspace_bytes(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], kind)
    assert 0 < need <= xp.xp_conv2d_nchw_static_max_bytes()
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    dx, dw = dev(x.reshape(-1)), dev(w.reshape(-1))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    a = torch.full((N, Cout, P, Q), float("nan"), device="cuda")
    b = torch.full((N, Cout, P, Q), float("nan"), device="cuda")
    xp.xp_conv2d_nchw(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], dx, dw, a, ws, in_type=kind, w_type=kind)
    xp.xp_conv2d_nchw_static(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], dx, dw, b, in_type=kind, w_type=kind)
    torch.cuda.synchronize()
    ref = oracle.conv2d_nchw(x, w, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S, stride=stride, pad=pad)
    return a.cpu().numpy(), b.cpu().numpy(), ref


@pytest.mark.parametrize("kind", ["bf16", "f32"])
def test_static_matches_workspace_entry_two_calls(xp, oracle, kind):
    """Two calls in a row, the second with a smaller input: what the first left in the buffer must not matter."""
    big = (3, 20, 18, 128, 96, 3, 3, (1, 1), (1, 1))
    small = (1, 7, 9, 64, 40, 3, 2, (2, 1), (1, 0))
    for seed, case in ((21, big), (22, small)):
        a, b, ref = _both(xp, oracle, kind, *case, seed)
        assert np.array_equal(a, b), f"static and workspace entry points differ: {kind} {case}"
        check_float(b, ref, f"conv nchw static {kind} {case}")


def test_static_rejects_more_than_its_buffer(xp):
    import torch
    # 64 x 128 x 64 x 64 fp32 activations alone are 128 MiB
    N, H, W, Cin, Cout = 64, 64, 64, 128, 8
    assert xp.xp_conv2d_nchw_workspace_bytes(N, H, W, Cin, Cout, 1, 1, 1, 1, 0, 0, "f32") > xp.xp_conv2d_nchw_static_max_bytes()
    x = torch.zeros(16, device="cuda")           # never read: the size check comes before any launch
    out = torch.zeros(16, device="cuda")
    with pytest.raises(xp.XpError) as e:
        xp.xp_conv2d_nchw_static(N, H, W, Cin, Cout, 1, 1, 1, 1, 0, 0, x, x, out, in_type="f32", w_type="f32")
    assert e.value.status == 2


def test_static_degenerate(xp):
    import torch
    x = torch.zeros(16, device="cuda")
    out = torch.zeros(16, device="cuda")
    xp.xp_conv2d_nchw_static(0, 4, 4, 8, 8, 3, 3, 1, 1, 1, 1, x, x, out, in_type="f32", w_type="f32")       # empty batch
    xp.xp_conv2d_nchw_static(1, 1, 1, 8, 8, 3, 3, 1, 1, 0, 0, x, x, out, in_type="f32", w_type="f32")       # image smaller than the filter
