"""Pins for the CPU oracle's memory-bound operators (Table 5 of the paper names them: Softmax,
LayerNorm, RMSNorm, ReLU, GeLU, Sigmoid, Sign, Add, Max/Avg/Min/SumPool; it prints no definition).

Closed forms, invariants and reductions to numpy / scipy routines, each aimed at a plausible mistake
(wrong axis, sample instead of population variance, missing eps, tanh-GELU for erf-GELU, padding
counted in the average, row pitch ignored).
"""
import math

import numpy as np
import pytest
from scipy.special import erf, expit, softmax

from paper_2505_02146_amd import inputs


def _rand(shape, tid, seed=21, sigma=1.0):
    return inputs.normal(shape, seed, tid, sigma).astype(np.float32)


def _pitched(m, ld, fill=np.nan):
    buf = np.full((m.shape[0], ld), fill, dtype=m.dtype)
    buf[:, :m.shape[1]] = m
    return buf.reshape(-1)


# ------------------------------------------------------------------------------------------ softmax

def test_softmax_constant_rows_and_row_sums(oracle):
    x = np.full((3, 7), 2.5, np.float32)
    np.testing.assert_allclose(oracle.softmax(x, rows=3, cols=7), 1.0 / 7.0, rtol=1e-15)
    y = oracle.softmax(_rand((6, 11), 1), rows=6, cols=11)
    assert (y > 0).all()
    np.testing.assert_allclose(y.sum(axis=1), 1.0, rtol=1e-14)       # rows, not columns, sum to one
    assert not np.allclose(y.sum(axis=0), 1.0)


def test_softmax_two_columns_is_the_logistic_function(oracle):
    x = _rand((9, 2), 1)
    y = oracle.softmax(x, rows=9, cols=2)
    np.testing.assert_allclose(y[:, 0], expit(x[:, 0].astype(np.float64) - x[:, 1].astype(np.float64)), rtol=1e-13)


def test_softmax_matches_scipy_with_pitch_bf16_and_huge_values(oracle):
    x = inputs.to_bf16_bits(_rand((5, 13), 1, sigma=30.0))
    buf = _pitched(x, 16, 0x7FC0)
    y = oracle.softmax(buf, rows=5, cols=13, ldx=16)
    np.testing.assert_allclose(y, softmax(inputs.bf16_bits_to_f32(x).astype(np.float64), axis=1), rtol=1e-12, atol=1e-300)
    big = np.array([[1e30, -1e30, 1e30]], np.float32)
    np.testing.assert_allclose(oracle.softmax(big, rows=1, cols=3), [[0.5, 0.0, 0.5]], rtol=1e-15)


def test_softmax_ignores_a_common_shift(oracle):
    x = _rand((4, 9), 1)
    a = oracle.softmax(x, rows=4, cols=9)
    b = oracle.softmax((x + np.float32(8.0)).astype(np.float32), rows=4, cols=9)    # x + 8 is rounded to fp32
    np.testing.assert_allclose(a, b, rtol=1e-5)


# ---------------------------------------------------------------------------------------- layernorm

def test_layernorm_hand_case_and_moments(oracle):
    x = np.array([[1.0, 2.0, 3.0, 4.0]], np.float32)
    eps = 1e-5
    y = oracle.layernorm(x, rows=1, cols=4, eps=eps)
    np.testing.assert_allclose(y[0], (np.array([1.0, 2.0, 3.0, 4.0]) - 2.5) / math.sqrt(1.25 + eps), rtol=1e-15)
    x = _rand((7, 33), 1, sigma=3.0) + 5.0
    eps = 1.0                                                         # large, so that the variance itself shows in the output
    y = oracle.layernorm(x, rows=7, cols=33, eps=eps)
    np.testing.assert_allclose(y.mean(axis=1), 0.0, atol=1e-14)
    var = x.astype(np.float64).var(axis=1)                            # population variance (ddof = 0)
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    sample = x.astype(np.float64).var(axis=1, ddof=1)
    assert not np.allclose(y.var(axis=1), var / (sample + eps), rtol=1e-3)


def test_layernorm_matches_numpy_with_gamma_beta_and_pitch(oracle):
    rows, cols, ld = 5, 19, 24
    x, g, b = _rand((rows, cols), 1), _rand((cols,), 2), _rand((cols,), 3)
    y = oracle.layernorm(_pitched(x, ld), rows=rows, cols=cols, gamma=g, beta=b, eps=1e-3, ldx=ld)
    xd = x.astype(np.float64)
    expect = (xd - xd.mean(axis=1, keepdims=True)) / np.sqrt(xd.var(axis=1, keepdims=True) + 1e-3) * g + b
    np.testing.assert_allclose(y, expect, rtol=1e-12, atol=1e-14)
    # beta alone shifts, gamma alone scales
    y0 = oracle.layernorm(x, rows=rows, cols=cols, eps=1e-3)
    np.testing.assert_allclose(oracle.layernorm(x, rows=rows, cols=cols, beta=b, eps=1e-3), y0 + b, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.layernorm(x, rows=rows, cols=cols, gamma=g, eps=1e-3), y0 * g, rtol=1e-13, atol=1e-15)


def test_layernorm_is_invariant_under_affine_maps_of_the_input_when_eps_is_zero(oracle):
    x = _rand((3, 16), 1)
    a = oracle.layernorm(x, rows=3, cols=16, eps=0.0)
    b = oracle.layernorm((2.0 * x + 3.0).astype(np.float32), rows=3, cols=16, eps=0.0)
    np.testing.assert_allclose(a, b, rtol=2e-5, atol=2e-6)             # 2x + 3 is rounded to fp32
    c = oracle.layernorm((-x).astype(np.float32), rows=3, cols=16, eps=0.0)
    np.testing.assert_allclose(c, -a, rtol=1e-14)


# ------------------------------------------------------------------------------------------ rmsnorm

def test_rmsnorm_hand_cases(oracle):
    x = np.array([[3.0, 4.0]], np.float32)
    np.testing.assert_allclose(oracle.rmsnorm(x, rows=1, cols=2, eps=0.0)[0], np.array([3.0, 4.0]) / math.sqrt(12.5), rtol=1e-15)
    c = np.full((2, 5), -2.0, np.float32)
    np.testing.assert_allclose(oracle.rmsnorm(c, rows=2, cols=5, eps=0.5), -2.0 / math.sqrt(4.5), rtol=1e-15)
    # the mean is NOT subtracted (that would be layernorm): a constant row does not map to zero
    assert abs(oracle.rmsnorm(c, rows=2, cols=5, eps=0.0)[0, 0] + 1.0) < 1e-15


def test_rmsnorm_matches_numpy_and_scales(oracle):
    rows, cols, ld = 4, 21, 32
    x, g = _rand((rows, cols), 1), _rand((cols,), 2)
    y = oracle.rmsnorm(_pitched(x, ld), rows=rows, cols=cols, gamma=g, eps=1e-6, ldx=ld)
    xd = x.astype(np.float64)
    np.testing.assert_allclose(y, xd / np.sqrt((xd * xd).mean(axis=1, keepdims=True) + 1e-6) * g, rtol=1e-12)
    a = oracle.rmsnorm(x, rows=rows, cols=cols, eps=0.0)
    b = oracle.rmsnorm((-4.0 * x).astype(np.float32), rows=rows, cols=cols, eps=0.0)      # exact scaling by a power of two
    np.testing.assert_allclose(b, -a, rtol=1e-14)
    np.testing.assert_allclose((a * a).mean(axis=1), 1.0, rtol=1e-13)                    # unit mean square


# --------------------------------------------------------------------------------------- pointwise

def test_unary_closed_forms(oracle):
    x = np.array([-3.5, -1.0, -0.0, 0.0, 0.25, 2.0, 40.0, -40.0], np.float32)
    np.testing.assert_array_equal(oracle.unary("relu", x), [0, 0, 0, 0, 0.25, 2.0, 40.0, 0])
    np.testing.assert_array_equal(oracle.unary("sign", x), [-1, -1, 0, 0, 1, 1, 1, -1])
    s = oracle.unary("sigmoid", x)
    assert s[3] == 0.5
    np.testing.assert_allclose(s + oracle.unary("sigmoid", -x), 1.0, rtol=1e-15)
    np.testing.assert_allclose(s, expit(x.astype(np.float64)), rtol=1e-14)
    g = oracle.unary("gelu", x)
    assert g[3] == 0.0
    np.testing.assert_allclose(g - oracle.unary("gelu", -x), x.astype(np.float64), rtol=1e-14, atol=1e-16)   # gelu(x) - gelu(-x) = x
    np.testing.assert_allclose(g, 0.5 * x.astype(np.float64) * (1.0 + erf(x.astype(np.float64) / math.sqrt(2.0))), rtol=1e-14)
    # the erf form, not the tanh approximation (they differ by 1e-4 at x = 2)
    tanh_form = 0.5 * 2.0 * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (2.0 + 0.044715 * 8.0)))
    assert abs(g[5] - tanh_form) > 5e-5 and abs(g[5] - 1.9544997361036416) < 1e-13


def test_unary_on_bf16_and_add(oracle):
    x = inputs.to_bf16_bits(_rand((3, 17), 1))
    xf = inputs.bf16_bits_to_f32(x).astype(np.float64)
    np.testing.assert_allclose(oracle.unary("gelu", x), 0.5 * xf * (1.0 + erf(xf / math.sqrt(2.0))), rtol=1e-14)
    a, b = _rand((4, 9), 1), _rand((4, 9), 2)
    np.testing.assert_array_equal(oracle.add(a, b), a.astype(np.float64) + b.astype(np.float64))
    ones = np.ones(5, np.float32)
    np.testing.assert_array_equal(oracle.add(ones, (2 * ones).astype(np.float32)), 3.0)


# ------------------------------------------------------------------------------------------ pooling

def test_pooling_all_ones_counts_the_positions_inside(oracle):
    N, H, W, C = 1, 4, 5, 2
    x = np.ones((N, H, W, C), np.float32)
    kw = dict(N=N, H=H, W=W, C=C, R=3, S=3, stride=(1, 1), pad=(1, 1))
    for op in ("max", "min", "avg"):
        np.testing.assert_array_equal(oracle.pool2d_nhwc(op, x, **kw), 1.0)          # padding is not averaged in
    s = oracle.pool2d_nhwc("sum", x, **kw)
    assert s.shape == (1, 4, 5, 2)
    assert s[0, 0, 0, 0] == 4 and s[0, 0, 2, 1] == 6 and s[0, 1, 2, 0] == 9 and s[0, 3, 4, 1] == 4


def test_pooling_whole_image_window_and_tiles_match_numpy(oracle):
    N, H, W, C = 2, 6, 8, 3
    x = _rand((N, H, W, C), 1)
    xd = x.astype(np.float64)
    for op, fn in (("max", np.max), ("min", np.min), ("sum", np.sum), ("avg", np.mean)):
        y = oracle.pool2d_nhwc(op, x, N=N, H=H, W=W, C=C, R=H, S=W)
        np.testing.assert_allclose(y[:, 0, 0, :], fn(xd, axis=(1, 2)), rtol=1e-13)
        # non-overlapping 2 x 4 tiles: a reshape does the same
        y = oracle.pool2d_nhwc(op, x, N=N, H=H, W=W, C=C, R=2, S=4, stride=(2, 4))
        np.testing.assert_allclose(y, fn(xd.reshape(N, 3, 2, 2, 4, C), axis=(2, 4)), rtol=1e-13)


def test_pooling_window_placement_and_negative_maxima(oracle):
    # a single non-zero pixel shows which outputs see it: rows p with p*2 - 1 <= 3 <= p*2 + 1, likewise columns
    N, H, W, C = 1, 7, 7, 1
    x = np.zeros((N, H, W, C), np.float32)
    x[0, 3, 4, 0] = 5.0
    y = oracle.pool2d_nhwc("sum", x, N=N, H=H, W=W, C=C, R=3, S=3, stride=(2, 2), pad=(1, 1))
    expect = np.zeros((4, 4))
    expect[1:3, 2] = 5.0               # rows 1, 2 (windows 1..3 and 3..5), column 2 (window 3..5)
    np.testing.assert_array_equal(y[0, :, :, 0], expect)
    # all-negative image: a maximum over the positions inside is negative, padding does not act as a zero
    neg = np.full((1, 3, 3, 1), -2.0, np.float32)
    np.testing.assert_array_equal(oracle.pool2d_nhwc("max", neg, N=1, H=3, W=3, C=1, R=3, S=3, pad=(1, 1)), -2.0)
    np.testing.assert_array_equal(oracle.pool2d_nhwc("min", -neg, N=1, H=3, W=3, C=1, R=3, S=3, pad=(1, 1)), 2.0)


def test_bad_arguments_are_refused(oracle):
    x = np.zeros(8, np.float32)
    with pytest.raises(ValueError):
        oracle.softmax(x, rows=2, cols=4, ldx=3)
    with pytest.raises(ValueError):
        oracle.pool2d_nhwc("max", x, N=1, H=2, W=2, C=2, R=0, S=1)
    assert oracle.softmax(x, rows=0, cols=4).shape == (0, 4)


# --------------------------------------------------------------------------------- depthwise conv

def test_depthwise_is_the_full_convolution_with_a_diagonal_filter(oracle):
    # w_full(k,r,s,c) = w(c,r,s) if k == c else 0 turns the (already pinned) dense convolution into the depthwise one
    N, H, W, C, R, S = 2, 6, 7, 5, 3, 2
    x = _rand((N, H, W, C), 1)
    w_crs = _rand((C, R, S), 2)
    full = np.zeros((C, R, S, C), np.float32)
    for c in range(C):
        full[c, :, :, c] = w_crs[c]
    kw = dict(stride=(2, 1), pad=(1, 1))
    expect = oracle.conv2d_nhwc(x, full, N=N, H=H, W=W, Cin=C, Cout=C, R=R, S=S, filter_layout="krsc", **kw)
    got = oracle.depthwise_conv2d_nhwc(x, w_crs, N=N, H=H, W=W, C=C, R=R, S=S, filter_layout="krsc", **kw)
    np.testing.assert_allclose(got, expect, rtol=1e-14, atol=1e-15)
    # the channel-minor filter layout holds the same numbers transposed
    w_rsc = np.ascontiguousarray(w_crs.transpose(1, 2, 0))
    np.testing.assert_array_equal(oracle.depthwise_conv2d_nhwc(x, w_rsc, N=N, H=H, W=W, C=C, R=R, S=S, filter_layout="rsck", **kw), got)


def test_depthwise_closed_forms(oracle):
    N, H, W, C = 1, 5, 6, 3
    x = _rand((N, H, W, C), 1)
    delta = np.zeros((3, 3, C), np.float32)
    delta[1, 1, :] = [1.0, 2.0, -1.0]                      # centre tap, a different gain per channel
    y = oracle.depthwise_conv2d_nhwc(x, delta, N=N, H=H, W=W, C=C, R=3, S=3, pad=(1, 1))
    np.testing.assert_array_equal(y, x.astype(np.float64) * np.array([1.0, 2.0, -1.0]))
    ones = np.ones((N, H, W, C), np.float32)
    y = oracle.depthwise_conv2d_nhwc(ones, np.ones((3, 3, C), np.float32), N=N, H=H, W=W, C=C, R=3, S=3, pad=(1, 1))
    assert y[0, 0, 0, 0] == 4 and y[0, 0, 3, 1] == 6 and y[0, 2, 2, 2] == 9
    # channels do not mix: changing channel 0 of the input leaves the other outputs alone
    x2 = x.copy()
    x2[..., 0] += 1.0
    w = _rand((3, 3, C), 2)
    a = oracle.depthwise_conv2d_nhwc(x, w, N=N, H=H, W=W, C=C, R=3, S=3, pad=(1, 1))
    b = oracle.depthwise_conv2d_nhwc(x2, w, N=N, H=H, W=W, C=C, R=3, S=3, pad=(1, 1))
    np.testing.assert_array_equal(a[..., 1:], b[..., 1:])
    assert not np.allclose(a[..., 0], b[..., 0])


# ------------------------------------------------------------------------------------- NCHW conv

def test_nchw_convolution_is_the_nhwc_one_on_transposed_data(oracle):
    N, H, W, Cin, Cout, R, S = 2, 6, 5, 3, 4, 3, 2
    x = _rand((N, Cin, H, W), 1)
    w = _rand((Cout, Cin, R, S), 2)
    kw = dict(stride=(2, 1), pad=(1, 2))
    got = oracle.conv2d_nchw(x, w, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S, **kw)
    x_nhwc = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    w_krsc = np.ascontiguousarray(w.transpose(0, 2, 3, 1))
    expect = oracle.conv2d_nhwc(x_nhwc, w_krsc, N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=S, filter_layout="krsc", **kw)
    np.testing.assert_allclose(got, expect.transpose(0, 3, 1, 2), rtol=1e-13, atol=1e-15)    # the channel sum runs in another order


def test_nchw_convolution_closed_forms(oracle):
    N, H, W, C = 1, 4, 5, 3
    x = _rand((N, C, H, W), 1)
    delta = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        delta[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(oracle.conv2d_nchw(x, delta, N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, pad=(1, 1)), x.astype(np.float64))
    # shifted delta: out[p, q] = in[p - 1, q - 1] with a zero border (correlation, not convolution)
    shift = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        shift[c, c, 0, 0] = 1.0
    y = oracle.conv2d_nchw(x, shift, N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, pad=(1, 1))
    np.testing.assert_array_equal(y[0, :, 1:, 1:], x[0, :, :-1, :-1].astype(np.float64))
    assert (y[0, :, 0, :] == 0).all() and (y[0, :, :, 0] == 0).all()
    ones = oracle.conv2d_nchw(np.ones((1, 2, 4, 4), np.float32), np.ones((1, 2, 3, 3), np.float32), N=1, H=4, W=4, Cin=2, Cout=1,
                              R=3, S=3, pad=(1, 1))
    assert ones[0, 0, 0, 0] == 8 and ones[0, 0, 0, 1] == 12 and ones[0, 0, 1, 1] == 18
