"""Memory-bound operators on the GPU against the CPU oracle, through the C ABI.

fp32 outputs: the two gates of the other floating-point operators plus the 1e-4 bound on the relative
Frobenius error (fp32 arithmetic on exact inputs).  bf16 outputs are a rounding decision: the GPU
rounds its fp32 result to nearest even, the expectation is the oracle's fp64 result rounded the same
way; the two may differ by one bf16 unit where the fp32 and fp64 values straddle a rounding
boundary, which must be rare (< 2 % of the elements) and never more than one unit (values whose
absolute error is below 1e-5 (1 + |ref|), i.e. inside fp32 noise, are exempt from the unit count).
"""
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
    return m


def _gen(kind, shape, tid, sigma=1.0, seed=31):
    a = inputs.normal(shape, seed, tid, sigma).astype(np.float32)
    return inputs.to_bf16_bits(a) if kind == "bf16" else a


def _out(kind, n, fill):
    import torch
    if kind == "bf16":
        return torch.full((n,), fill, dtype=torch.bfloat16, device="cuda")
    return torch.full((n,), fill, dtype=torch.float32, device="cuda")


def _host(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _check(got, ref, what):
    """got: float32 array, or uint16 bf16 bits; ref: float64."""
    if got.dtype == np.uint16:
        want = inputs.to_bf16_bits(ref.astype(np.float32))
        g, w = got.astype(np.int32).reshape(-1), want.astype(np.int32).reshape(-1)
        # sign-magnitude bit patterns -> a monotone integer scale
        g = np.where(g & 0x8000, -(g & 0x7FFF), g)
        w = np.where(w & 0x8000, -(w & 0x7FFF), w)
        d = np.abs(g - w)
        # near zero (results of a cancellation, such as x - mean) a bf16 unit is far below the noise of
        # the fp32 arithmetic itself: there the absolute error is what can be asked for
        near = np.abs(inputs.bf16_bits_to_f32(got).astype(np.float64).reshape(-1) - ref.reshape(-1)) <= 1e-5 * (1.0 + np.abs(ref.reshape(-1)))
        worst = d[~near].max() if (~near).any() else 0
        assert worst <= 1, f"{what}: bf16 output off by {worst} units"
        assert (d != 0).mean() < 0.02, f"{what}: {100 * (d != 0).mean():.2f} % of bf16 outputs differ from the rounded oracle"
    else:
        check_float(got, ref, what)


def _pitched(m, ld, fill):
    buf = np.full((m.shape[0], ld), fill, dtype=m.dtype)
    buf[:, :m.shape[1]] = m
    return buf.reshape(-1)


ROW_SHAPES = [  # rows, cols, pitch padding (elements)
    (1, 8, 0), (3, 5, 0), (4, 64, 8), (7, 520, 0), (33, 4096, 0), (5, 8200, 8), (2, 40000, 0), (6, 1000, 24), (9, 16392, 0),
    (300, 256, 0),
]


@pytest.mark.parametrize("op", ["softmax", "layernorm", "rmsnorm"])
@pytest.mark.parametrize("kinds", [("f32", "f32"), ("bf16", "f32"), ("bf16", "bf16"), ("f32", "bf16")])
def test_row_operators(xp, oracle, op, kinds):
    kin, kout = kinds
    nan = 0x7FC0 if kin == "bf16" else np.nan
    for rows, cols, pad in ROW_SHAPES:
        x = _gen(kin, (rows, cols), 1, sigma=2.0)
        g, b = _gen(kin, (cols,), 2), _gen(kin, (cols,), 3)
        ldx, ldy = cols + pad, cols + (pad // 2 if pad else 0)
        xb = _pitched(x, ldx, nan)
        y = _out(kout, rows * ldy, -3.0)
        if op == "softmax":
            xp.xp_softmax(rows, cols, dev(xb), ldx, y, ldy, x_type=kin)
            ref = oracle.softmax(xb, rows=rows, cols=cols, ldx=ldx)
        elif op == "layernorm":
            xp.xp_layernorm(rows, cols, dev(xb), ldx, dev(g), dev(b), 1e-5, y, ldy, x_type=kin)
            ref = oracle.layernorm(xb, rows=rows, cols=cols, gamma=g, beta=b, eps=1e-5, ldx=ldx)
        else:
            xp.xp_rmsnorm(rows, cols, dev(xb), ldx, dev(g), 1e-6, y, ldy, x_type=kin)
            ref = oracle.rmsnorm(xb, rows=rows, cols=cols, gamma=g, eps=1e-6, ldx=ldx)
        got = _host(y).reshape(rows, ldy)
        _check(np.ascontiguousarray(got[:, :cols]), ref, f"{op} {kinds} {(rows, cols, pad)}")
        if ldy > cols:                                   # nothing written between the rows
            pad_vals = got[:, cols:]
            assert (pad_vals == (0xC040 if kout == "bf16" else -3.0)).all()


def test_norms_without_gamma_beta_and_in_place(xp, oracle):
    rows, cols = 40, 768
    x = _gen("f32", (rows, cols), 1, sigma=3.0)
    y = _out("f32", rows * cols, 0.0)
    xp.xp_layernorm(rows, cols, dev(x.reshape(-1)), cols, None, None, 1e-5, y, cols)
    check_float(_host(y).reshape(rows, cols), oracle.layernorm(x, rows=rows, cols=cols, eps=1e-5), "layernorm plain")
    xp.xp_rmsnorm(rows, cols, dev(x.reshape(-1)), cols, None, 1e-6, y, cols)
    check_float(_host(y).reshape(rows, cols), oracle.rmsnorm(x, rows=rows, cols=cols, eps=1e-6), "rmsnorm plain")
    d = dev(x.reshape(-1).copy())
    xp.xp_softmax(rows, cols, d, cols, d, cols)          # in place
    check_float(d.cpu().numpy().reshape(rows, cols), oracle.softmax(x, rows=rows, cols=cols), "softmax in place")


def test_softmax_of_large_and_equal_values(xp, oracle):
    x = np.array([[1e30, -1e30, 1e30, 0.0], [5.0, 5.0, 5.0, 5.0], [-80.0, 0.0, 80.0, 79.0]], np.float32)
    y = _out("f32", 12, -1.0)
    xp.xp_softmax(3, 4, dev(x.reshape(-1)), 4, y, 4)
    check_float(_host(y).reshape(3, 4), oracle.softmax(x, rows=3, cols=4), "softmax extremes")


@pytest.mark.parametrize("op", ["relu", "gelu", "sigmoid", "sign"])
@pytest.mark.parametrize("kinds", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "bf16")])
def test_unary(xp, oracle, op, kinds):
    kin, kout = kinds
    for n in (1, 7, 1000, (1 << 20) + 3):
        x = _gen(kin, (n,), 1, sigma=3.0)
        if n >= 7:                                       # the special points
            sp = np.array([0.0, -0.0, 1.0, -1.0, 30.0, -30.0, 0.5], np.float32)
            x[:7] = inputs.to_bf16_bits(sp) if kin == "bf16" else sp
        y = _out(kout, n, 9.0)
        xp.xp_unary(op, n, dev(x), y, x_type=kin)
        _check(_host(y), oracle.unary(op, x), f"{op} {kinds} n={n}")
    # pointers that are only element-aligned take the scalar path
    n = 1001
    x = _gen(kin, (n + 1,), 1)
    dx, y = dev(x), _out(kout, n + 1, 9.0)
    xp.xp_unary(op, n, dx[1:], y[1:], x_type=kin)
    _check(_host(y)[1:], oracle.unary(op, x[1:].copy()), f"{op} {kinds} unaligned")
    assert _host(y)[0] == (0x4110 if kout == "bf16" else 9.0)


@pytest.mark.parametrize("kinds", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
def test_add(xp, oracle, kinds):
    kin, kout = kinds
    for n in (5, 4096, 100003):
        a, b = _gen(kin, (n,), 1), _gen(kin, (n,), 2)
        y = _out(kout, n, 0.0)
        xp.xp_add(n, dev(a), dev(b), y, x_type=kin)
        _check(_host(y), oracle.add(a, b), f"add {kinds} n={n}")
    if kin == kout:
        a, b = _gen(kin, (300,), 1), _gen(kin, (300,), 2)
        import torch
        d = dev(a.copy())
        d = d.view(torch.bfloat16) if kin == "bf16" else d
        xp.xp_add(300, d, dev(b), d, x_type=kin)         # in place
        _check(_host(d), oracle.add(a, b), "add in place")


POOL_CASES = [  # N, H, W, C, R, S, stride, pad
    (2, 8, 8, 16, 2, 2, (2, 2), (0, 0)),
    (1, 7, 9, 8, 3, 3, (2, 1), (1, 1)),
    (1, 5, 5, 3, 3, 3, (1, 1), (1, 1)),                  # 3 channels: scalar path
    (2, 12, 12, 64, 3, 3, (2, 2), (1, 1)),
    (1, 6, 6, 8, 6, 6, (1, 1), (0, 0)),                  # one window: global pooling
    (1, 4, 4, 8, 2, 2, (3, 3), (2, 2)),                  # windows entirely in the padding: zeros
]


@pytest.mark.parametrize("op", ["max", "avg", "min", "sum"])
@pytest.mark.parametrize("kinds", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
def test_pooling(xp, oracle, op, kinds):
    kin, kout = kinds
    for (N, H, W, C, R, S, stride, pad) in POOL_CASES:
        x = _gen(kin, (N, H, W, C), 1)
        if op == "max":
            x = _gen(kin, (N, H, W, C), 1) if kin == "bf16" else (x - 5.0).astype(np.float32)   # negative maxima
        ref = oracle.pool2d_nhwc(op, x, N=N, H=H, W=W, C=C, R=R, S=S, stride=stride, pad=pad)
        y = _out(kout, ref.size, 7.0)
        xp.xp_pool2d_nhwc(op, N, H, W, C, R, S, stride[0], stride[1], pad[0], pad[1], dev(x.reshape(-1)), y, x_type=kin)
        _check(_host(y).reshape(ref.shape), ref, f"{op}pool {kinds} {(N, H, W, C, R, S, stride, pad)}")


def test_validation_on_the_device_side_of_the_abi(xp):
    import torch
    x = torch.zeros(64, device="cuda")
    for call in (lambda: xp.xp_softmax(2, 8, x, 4, x, 8), lambda: xp.xp_layernorm(2, 8, x, 8, None, None, -1.0, x, 8),
                 lambda: xp.xp_rmsnorm(2, 8, x, 8, None, float("nan"), x, 8)):
        with pytest.raises(xp.XpError):
            call()
    xp.xp_softmax(0, 8, None, 8, None, 8, x_type="f32", y_type="f32")    # empty: nothing to do


def test_layernorm_and_softmax_workloads_full_size(xp, oracle):
    """The shapes the benchmark times; rows sampled for the oracle."""
    import torch
    rng = np.random.default_rng(3)
    rows, cols = 16384, 4096
    x = _gen("bf16", (rows, cols), 1, sigma=1.5)
    g, b = _gen("bf16", (cols,), 2), _gen("bf16", (cols,), 3)
    y = _out("bf16", rows * cols, 0.0)
    xp.xp_layernorm(rows, cols, dev(x.reshape(-1)), cols, dev(g), dev(b), 1e-5, y, cols, x_type="bf16")
    pick = np.sort(rng.choice(rows, 256, replace=False))
    pick[0], pick[-1] = 0, rows - 1
    got = _host(y).reshape(rows, cols)[pick]
    _check(np.ascontiguousarray(got), oracle.layernorm(np.ascontiguousarray(x[pick]), rows=len(pick), cols=cols, gamma=g, beta=b,
                                                       eps=1e-5), "layernorm workload")
    xp.xp_rmsnorm(rows, cols, dev(x.reshape(-1)), cols, dev(g), 1e-6, y, cols, x_type="bf16")
    got = _host(y).reshape(rows, cols)[pick]
    _check(np.ascontiguousarray(got), oracle.rmsnorm(np.ascontiguousarray(x[pick]), rows=len(pick), cols=cols, gamma=g, eps=1e-6),
           "rmsnorm workload")
    rows, cols = 96 * 512, 512
    s = _gen("f32", (rows, cols), 1, sigma=1.0)
    ys = _out("f32", rows * cols, 0.0)
    xp.xp_softmax(rows, cols, dev(s.reshape(-1)), cols, ys, cols)
    check_float(_host(ys).reshape(rows, cols), oracle.softmax(s, rows=rows, cols=cols), "softmax workload")


DW_CASES = [  # N, H, W, C, R, S, stride, pad
    (2, 8, 8, 16, 3, 3, (1, 1), (1, 1)),
    (1, 9, 7, 8, 3, 3, (2, 2), (1, 1)),
    (1, 6, 6, 5, 3, 3, (1, 1), (1, 1)),                  # 5 channels: scalar path
    (2, 10, 12, 32, 5, 3, (2, 1), (2, 1)),               # non-square window: general loop
    (1, 14, 14, 64, 3, 3, (1, 1), (0, 0)),
    (1, 3, 3, 8, 1, 1, (1, 1), (0, 0)),                  # 1 x 1: a per-channel scale
    # the LDS-tiled 3 x 3 stride-1 kernel (channel-minor weights): output tiles cut by the right and bottom
    # edges, a last block of channel chunks that is partly empty, with and without padding
    (2, 19, 37, 72, 3, 3, (1, 1), (1, 1)),
    (1, 20, 40, 64, 3, 3, (1, 1), (0, 0)),
    (1, 8, 16, 8, 3, 3, (1, 1), (1, 1)),                 # exactly one tile, one chunk
]


@pytest.mark.parametrize("layout", ["rsck", "krsc"])
@pytest.mark.parametrize("kinds", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
def test_depthwise_conv(xp, oracle, layout, kinds):
    kin, kout = kinds
    for (N, H, W, C, R, S, stride, pad) in DW_CASES:
        x = _gen(kin, (N, H, W, C), 1)
        w = _gen(kin, (R, S, C) if layout == "rsck" else (C, R, S), 2, sigma=0.3)
        ref = oracle.depthwise_conv2d_nhwc(x, w, N=N, H=H, W=W, C=C, R=R, S=S, stride=stride, pad=pad, filter_layout=layout)
        y = _out(kout, ref.size, 7.0)
        xp.xp_depthwise_conv2d_nhwc(N, H, W, C, R, S, stride[0], stride[1], pad[0], pad[1], dev(x.reshape(-1)),
                                    dev(w.reshape(-1)), layout, y, x_type=kin, w_type=kin)
        _check(_host(y).reshape(ref.shape), ref, f"depthwise {layout} {kinds} {(N, H, W, C, R, S, stride, pad)}")


def test_depthwise_workload_full_size(xp, oracle):
    """A MobileNet-like stage: 32 x 112 x 112 x 64, 3 x 3, stride 1, pad 1, bf16 in and out."""
    N, H, W, C = 32, 112, 112, 64
    x = _gen("bf16", (N, H, W, C), 1)
    w = _gen("bf16", (3, 3, C), 2, sigma=0.3)
    y = _out("bf16", N * H * W * C, 0.0)
    xp.xp_depthwise_conv2d_nhwc(N, H, W, C, 3, 3, 1, 1, 1, 1, dev(x.reshape(-1)), dev(w.reshape(-1)), "rsck", y,
                                x_type="bf16", w_type="bf16")
    got = _host(y).reshape(N, H, W, C)
    for n in (0, 17, 31):                                # three whole images
        ref = oracle.depthwise_conv2d_nhwc(np.ascontiguousarray(x[n:n + 1]), w, N=1, H=H, W=W, C=C, R=3, S=3, pad=(1, 1))
        _check(np.ascontiguousarray(got[n:n + 1]), ref, f"depthwise workload image {n}")
