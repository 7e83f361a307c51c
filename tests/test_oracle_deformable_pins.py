"""Pins for the CPU oracle's multi-scale deformable attention (Table 5 names the operator; the
definition is the one of Deformable DETR: bilinear samples of each feature level at fractional
positions, zero outside, weighted and summed).  Closed forms and a reduction to scipy's
`map_coordinates`, aimed at: x/y swapped, the half-pixel offset dropped, levels mis-addressed,
weights applied to the wrong point, border pixels clamped instead of zeroed."""
import numpy as np
from scipy.ndimage import map_coordinates

from paper_2505_02146_amd import inputs


def _rand(shape, tid, seed=41):
    return inputs.normal(shape, seed, tid).astype(np.float32)


def test_sampling_at_pixel_centres_returns_the_pixels(oracle):
    H, W, heads, d = 3, 5, 2, 4
    v = _rand((1, H * W, heads, d), 1)
    # one query per pixel, one level, one point with weight 1 at the centre of that pixel: (x + 0.5)/W, (y + 0.5)/H
    ys, xs = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    loc = np.zeros((1, H * W, heads, 1, 1, 2), np.float32)
    loc[0, :, :, 0, 0, 0] = ((xs.reshape(-1) + 0.5) / W)[:, None]
    loc[0, :, :, 0, 0, 1] = ((ys.reshape(-1) + 0.5) / H)[:, None]
    w = np.ones((1, H * W, heads, 1, 1), np.float32)
    out = oracle.deformable_attention(v, [(H, W)], loc, w, batch=1, Lq=H * W, heads=heads, d=d, points=1)
    np.testing.assert_allclose(out[0], v[0].astype(np.float64), rtol=1e-6, atol=1e-7)   # (x + 0.5)/W is rounded to fp32


def test_midpoints_average_and_borders_are_zero_padded(oracle):
    H, W = 2, 2
    v = np.array([1.0, 2.0, 3.0, 4.0], np.float32).reshape(1, 4, 1, 1)          # [[1, 2], [3, 4]]
    def at(x, y):
        loc = np.array([x, y], np.float32).reshape(1, 1, 1, 1, 1, 2)
        return oracle.deformable_attention(v, [(H, W)], loc, np.ones((1, 1, 1, 1, 1), np.float32), batch=1, Lq=1, heads=1, d=1,
                                           points=1)[0, 0, 0, 0]
    assert at(0.5, 0.5) == 2.5                      # the centre of the 2 x 2 map: mean of the four
    assert at(0.5, 0.25) == 1.5                     # between pixels (0,0) and (0,1): x is the width axis
    assert at(0.25, 0.5) == 2.0                     # between pixels (0,0) and (1,0)
    assert at(0.0, 0.25) == 0.5                     # half a pixel left of pixel (0,0): half of it, the rest is zero padding
    assert at(0.0, 0.0) == 0.25                     # the corner of the map: a quarter of pixel (0,0)
    assert at(-0.5, 0.5) == 0.0 and at(0.5, 1.5) == 0.0 and at(1.0, 1.0) == 1.0   # far outside: nothing; far corner: 4/4


def test_matches_scipy_interpolation_level_by_level(oracle):
    levels = [(6, 7), (3, 4), (2, 2)]
    heads, d, Lq, points, batch = 3, 5, 11, 4, 2
    S = sum(h * w for h, w in levels)
    v = _rand((batch, S, heads, d), 1)
    rng = np.random.default_rng(7)
    loc = rng.uniform(-0.15, 1.15, size=(batch, Lq, heads, len(levels), points, 2)).astype(np.float32)
    w = rng.uniform(0, 1, size=(batch, Lq, heads, len(levels), points)).astype(np.float32)
    out = oracle.deformable_attention(v, levels, loc, w, batch=batch, Lq=Lq, heads=heads, d=d, points=points)
    expect = np.zeros((batch, Lq, heads, d))
    start = 0
    for l, (H, W) in enumerate(levels):
        fmap = v[:, start:start + H * W].astype(np.float64).reshape(batch, H, W, heads, d)
        start += H * W
        x = loc[:, :, :, l, :, 0].astype(np.float64) * W - 0.5
        y = loc[:, :, :, l, :, 1].astype(np.float64) * H - 0.5
        for n in range(batch):
            for m in range(heads):
                for c in range(d):
                    s = map_coordinates(fmap[n, :, :, m, c], [y[n, :, m].reshape(-1), x[n, :, m].reshape(-1)], order=1,
                                        mode="grid-constant", cval=0.0).reshape(Lq, points)
                    expect[n, :, m, c] += (s * w[n, :, m, l].astype(np.float64)).sum(axis=1)
    np.testing.assert_allclose(out, expect, rtol=1e-12, atol=1e-13)


def test_constant_maps_and_linearity_in_the_weights(oracle):
    levels = [(4, 4), (2, 3)]
    heads, d, Lq, points = 2, 3, 5, 2
    S = sum(h * w for h, w in levels)
    rng = np.random.default_rng(8)
    loc = rng.uniform(0.3, 0.7, size=(1, Lq, heads, 2, points, 2)).astype(np.float32)    # well inside: no padding involved
    w = rng.uniform(0, 1, size=(1, Lq, heads, 2, points)).astype(np.float32)
    ones = np.ones((1, S, heads, d), np.float32)
    out = oracle.deformable_attention(ones, levels, loc, w, batch=1, Lq=Lq, heads=heads, d=d, points=points)
    np.testing.assert_allclose(out, np.broadcast_to(w.astype(np.float64).sum(axis=(3, 4))[..., None], out.shape), rtol=1e-12)
    v = _rand((1, S, heads, d), 1)
    a = oracle.deformable_attention(v, levels, loc, w, batch=1, Lq=Lq, heads=heads, d=d, points=points)
    b = oracle.deformable_attention(v, levels, loc, (2 * w).astype(np.float32), batch=1, Lq=Lq, heads=heads, d=d, points=points)
    np.testing.assert_allclose(b, 2 * a, rtol=1e-14)
    # a weight on one (level, point) only: the output is that single sample, so levels and points are not confused
    w1 = np.zeros_like(w)
    w1[..., 1, 0] = 1.0
    only = oracle.deformable_attention(v, levels, loc, w1, batch=1, Lq=Lq, heads=heads, d=d, points=points)
    H, W = levels[1]
    fmap = v[0, 16:].astype(np.float64).reshape(H, W, heads, d)
    for q in range(Lq):
        for m in range(heads):
            x, y = float(loc[0, q, m, 1, 0, 0]) * W - 0.5, float(loc[0, q, m, 1, 0, 1]) * H - 0.5
            for c in range(d):
                s = map_coordinates(fmap[:, :, m, c], [[y], [x]], order=1, mode="grid-constant", cval=0.0)[0]
                assert abs(only[0, q, m, c] - s) < 1e-12
