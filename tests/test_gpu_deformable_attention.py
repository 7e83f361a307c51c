"""Multi-scale deformable attention on the GPU against the CPU oracle, through the C ABI.

Positions are computed in fp32 on the GPU and in fp64 by the oracle; the bilinear sample is continuous
in the position (also across pixel boundaries and into the zero padding), so the difference is a few
fp32 units of the position times the local slope of the map: the gate is |err| <= 1e-4 (|ref| + 1),
a hundred times tighter than the contraction operators' gate.  bf16 outputs are compared after
widening, with the bf16 rounding step 2^-8 |ref| added.
"""
import numpy as np
import pytest

from paper_2505_02146_amd import inputs
from tests.helpers import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xp():
    import torch
    assert torch.cuda.is_available()
    from paper_2505_02146_amd import xp as m
    return m


def _case(batch, Lq, heads, d, levels, points, kind, seed, lo=-0.1, hi=1.1):
    S = sum(h * w for h, w in levels)
    v = inputs.normal((batch, max(S, 1), heads, d), seed, 1).astype(np.float32)[:, :S]
    v = np.ascontiguousarray(v)
    if kind == "bf16":
        v = inputs.to_bf16_bits(v)
    rng = np.random.default_rng(seed)
    loc = rng.uniform(lo, hi, size=(batch, Lq, heads, len(levels), points, 2)).astype(np.float32)
    w = rng.uniform(0, 1, size=(batch, Lq, heads, len(levels), points)).astype(np.float32)
    if w.size:
        w /= np.maximum(w.sum(axis=(3, 4), keepdims=True), 1e-6)          # as a softmax would leave them
    return v, loc, w


def _run(xp, batch, Lq, heads, d, levels, points, v, loc, w, kin, kout):
    import torch
    n = batch * Lq * heads * d
    out = torch.full((max(n, 1),), 7.0, device="cuda", dtype=torch.bfloat16 if kout == "bf16" else torch.float32)
    xp.xp_deformable_attention(batch, Lq, heads, d, points, dev(v.reshape(-1)) if v.size else None, levels,
                               dev(loc.reshape(-1)) if loc.size else None, dev(w.reshape(-1)) if w.size else None, out,
                               v_type=kin)
    torch.cuda.synchronize()
    return out[:n].float().cpu().numpy().astype(np.float64).reshape(batch, Lq, heads, d)


def _check(got, ref, kout, what):
    tol = 1e-4 * (np.abs(ref) + 1.0) + (2.0 ** -8 * np.abs(ref) if kout == "bf16" else 0.0)
    err = np.abs(got - ref)
    assert (err <= tol).all(), f"{what}: max excess {(err - tol).max():.3e} at {np.unravel_index((err - tol).argmax(), err.shape)}"


CASES = [  # batch, Lq, heads, d, levels, points
    (1, 1, 1, 8, [(4, 4)], 1),
    (2, 37, 3, 32, [(9, 13), (5, 7), (3, 3), (1, 2)], 4),          # the vectorised path, ragged maps
    (1, 300, 8, 32, [(16, 16), (8, 8)], 4),                        # more than one workgroup
    (2, 11, 2, 12, [(6, 5), (2, 2)], 3),                           # d = 12: 16-byte chunks for fp32, scalar for bf16
    (1, 9, 2, 5, [(4, 6)], 2),                                     # odd d: scalar path
    (1, 5, 1, 16, [(1, 1)], 8),                                    # a single pixel: everything is border
    (1, 4, 2, 8, [(3, 0), (2, 2)], 2),                             # an empty level contributes nothing
    # many queries per (image, head): the kernel that first copies the small levels into LDS
    (1, 4000, 2, 32, [(9, 13), (5, 7), (3, 3)], 4),                # all levels staged
    (2, 3001, 3, 16, [(40, 50), (7, 5), (0, 4), (2, 3)], 5),       # the largest level stays in global memory; ragged blocks
    (1, 2500, 1, 64, [(6, 6)], 1),
    (1, 50, 2, 16, [(5, 5), (3, 4)], 4),                           # four lanes a head for fp32, two for bf16
    (1, 3000, 2, 16, [(12, 12), (3, 4)], 4),                       # the same through LDS
]


@pytest.mark.parametrize("kinds", [("f32", "f32"), ("bf16", "f32"), ("bf16", "bf16"), ("f32", "bf16")])
def test_against_oracle(xp, oracle, kinds):
    kin, kout = kinds
    for i, (batch, Lq, heads, d, levels, points) in enumerate(CASES):
        v, loc, w = _case(batch, Lq, heads, d, levels, points, kin, 50 + i)
        ref = oracle.deformable_attention(v, levels, loc, w, batch=batch, Lq=Lq, heads=heads, d=d, points=points)
        got = _run(xp, batch, Lq, heads, d, levels, points, v, loc, w, kin, kout)
        _check(got, ref, kout, f"case {i} {kinds}")


@pytest.mark.parametrize("d,kind,points,Lq", [(8, "f32", 2, 30), (32, "bf16", 4, 30), (16, "f32", 4, 30), (16, "bf16", 4, 30),
                                              (32, "bf16", 4, 3000)])
def test_positions_far_outside_nan_and_exact_pixel_centres(xp, oracle, d, kind, points, Lq):
    """Every way of reading the points (any number, four a level, four a level shared among four lanes;
    from global memory and, with 3000 queries, from LDS).  Pixel (0,0), where the kernels point the
    fetches of a position outside the map, holds an infinity: it must not reach those sums."""
    levels, heads = [(5, 6)], 2
    v, loc, w = _case(1, Lq, heads, d, levels, points, kind, 71, lo=0.25, hi=1.1)      # no sample touches pixel (0,0)
    if kind == "bf16":
        v[0, 0] = 0x7F80
    else:
        v[0, 0] = np.inf
    loc[0, :10] = np.float32(3.0e9)                   # far outside: nothing
    loc[0, 10:12] = np.float32(-1.0e30)
    ys, xs = np.meshgrid(np.arange(5), np.arange(6), indexing="ij")
    centres = np.stack([(xs.reshape(-1) + 0.5) / 6, (ys.reshape(-1) + 0.5) / 5], axis=-1).astype(np.float32)
    loc[0, 12:30] = centres[12:30, None, None, None, :]              # pixels 12.. : not pixel (0,0)
    ref = oracle.deformable_attention(v, levels, loc, w, batch=1, Lq=Lq, heads=heads, d=d, points=points)
    assert np.isfinite(ref).all()
    got = _run(xp, 1, Lq, heads, d, levels, points, v, loc, w, kind, "f32")
    _check(got, ref, "f32", "far outside / centres")
    assert (got[0, :12] == 0).all()
    nan_loc = loc.copy()
    nan_loc[0, 3, 1, 0, :, 0] = np.nan                # NaN positions are skipped like those outside
    nan_loc[0, 20, 0, 0, 1, 1] = np.nan
    got2 = _run(xp, 1, Lq, heads, d, levels, points, v, nan_loc, w, kind, "f32")
    assert np.isfinite(got2).all() and (got2[0, 3, 1] == 0).all()
    keep = np.ones(got.shape, bool)
    keep[0, 3, 1] = keep[0, 20, 0] = False
    assert (got2[keep] == got[keep]).all()


def test_no_levels_or_points_write_zeros_and_empty_calls_write_nothing(xp):
    import torch
    out = torch.full((64,), 7.0, device="cuda")
    loc = torch.zeros(8, device="cuda")
    xp.xp_deformable_attention(1, 2, 2, 16, 0, None, [(4, 4)], None, None, out, v_type="f32")            # points == 0
    torch.cuda.synchronize()
    assert (out == 0).all()
    out.fill_(7.0)
    xp.xp_deformable_attention(1, 2, 2, 16, 3, None, [], loc, loc, out, v_type="f32")                    # no levels
    torch.cuda.synchronize()
    assert (out == 0).all()
    out.fill_(7.0)
    xp.xp_deformable_attention(0, 2, 2, 16, 3, None, [(4, 4)], None, None, out, v_type="f32")
    xp.xp_deformable_attention(1, 0, 2, 16, 3, None, [(4, 4)], None, None, out, v_type="f32")
    torch.cuda.synchronize()
    assert (out == 7.0).all()


def test_workload_full_size(xp, oracle):
    """A detection encoder layer: batch 8, four levels 64x64 .. 8x8 (5440 pixels, as many queries),
    8 heads of 32 channels, 4 points per level, bf16 values, fp32 output.  Sampled queries are
    checked against the oracle run on those queries alone."""
    levels = inputs.DEFORMABLE_WORKLOAD["levels"]
    batch, heads, d, points = (inputs.DEFORMABLE_WORKLOAD[k] for k in ("batch", "heads", "d", "points"))
    Lq = sum(h * w for h, w in levels)
    v, loc, w = inputs.deformable_attention_inputs(batch, Lq, heads, d, levels, points, seed=5)
    got = _run(xp, batch, Lq, heads, d, levels, points, v, loc, w, "bf16", "f32")
    rng = np.random.default_rng(0)
    for n in (0, 3, 7):
        qs = np.sort(rng.choice(Lq, size=200, replace=False))
        ref = oracle.deformable_attention(np.ascontiguousarray(v[n:n + 1]), levels, np.ascontiguousarray(loc[n:n + 1, qs]),
                                          np.ascontiguousarray(w[n:n + 1, qs]), batch=1, Lq=len(qs), heads=heads, d=d, points=points)
        _check(got[n:n + 1, qs], ref, "f32", f"workload image {n}")
