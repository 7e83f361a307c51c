"""The accuracy gates a floating-point result has to pass against the fp64 reference: every element within
1e-2 * (|ref| + 1) and a relative Frobenius error of at most 5e-3 (int8 -> int32 results are compared bit for
bit instead).  Shared by the tests, the smoke run and the benchmark; holds no operator arithmetic."""
from __future__ import annotations

import numpy as np

GATE_ELEM = 1e-2        # |err| <= GATE_ELEM * (|ref| + 1), elementwise
GATE_FRO = 5e-3         # ||gpu - ref||_F / ||ref||_F
# Second, tighter bound derived from the arithmetic: inputs are exact (bf16 or fp32 bit patterns
# shared with the reference), products of bf16 pairs are exact in fp32, so the only error is fp32
# accumulation of K terms: relative Frobenius error ~ sqrt(K) * 2^-24 (4e-6 at K = 4096).
# A dropped K step or a bf16-rounded accumulator would show up as 1e-3 or more.
TIGHT_FRO = 1e-4


def margins(gpu: np.ndarray, ref: np.ndarray):
    """(largest |err| / (|ref| + 1), relative Frobenius error); infinities if the output is not finite."""
    g = np.asarray(gpu, dtype=np.float64).reshape(-1)
    r = np.asarray(ref, dtype=np.float64).reshape(-1)
    if g.shape != r.shape or not np.all(np.isfinite(g)):
        return float("inf"), float("inf")
    if g.size == 0:
        return 0.0, 0.0
    worst = float(np.max(np.abs(g - r) / (np.abs(r) + 1.0)))
    nref = float(np.linalg.norm(r))
    fro = float(np.linalg.norm(g - r)) / nref if nref > 0 else float(np.linalg.norm(g - r))
    return worst, fro


def check_float(gpu: np.ndarray, ref: np.ndarray, what: str = "", tight: bool = True):
    """Asserts the two gates (and, with `tight`, the fp32-accumulation bound); returns the margins."""
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite output"
    worst, fro = margins(gpu, ref)
    assert worst <= GATE_ELEM, f"{what}: elementwise gate {worst:.3e} > {GATE_ELEM}"
    assert fro <= GATE_FRO, f"{what}: Frobenius gate {fro:.3e} > {GATE_FRO}"
    if tight:
        assert fro <= TIGHT_FRO, f"{what}: relative Frobenius error {fro:.3e} above the fp32-accumulation bound"
    return worst, fro
