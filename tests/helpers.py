"""Shared pieces of the GPU parity tests: device marshalling, gates, call wrappers."""
from __future__ import annotations

import numpy as np

GATE_ELEM = 1e-2        # |err| <= GATE_ELEM * (|ref| + 1), elementwise
GATE_FRO = 5e-3         # ||gpu - ref||_F / ||ref||_F
# Second, tighter bound derived from the arithmetic: inputs are exact (bf16 or fp32 bit patterns
# shared with the oracle), products of bf16 pairs are exact in fp32, so the only error is fp32
# accumulation of K terms: relative Frobenius error ~ sqrt(K) * 2^-24 (4e-6 at K = 4096).
# A dropped K step or a bf16-rounded accumulator would show up as 1e-3 or more.
TIGHT_FRO = 1e-4


def dev(a: np.ndarray, bf16: bool = False):
    """numpy host array -> torch tensor on cuda:0 (uint16 bf16 bits travel as int16)."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def store(mat: np.ndarray, layout: str, ld_pad: int = 0, fill=0):
    """Flat buffer holding logical matrix `mat` in `layout` with padded leading dimension."""
    rows, cols = mat.shape
    if layout == "row":
        ld = cols + ld_pad
        buf = np.full((rows, ld), fill, dtype=mat.dtype)
        buf[:, :cols] = mat
    else:
        ld = rows + ld_pad
        buf = np.full((cols, ld), fill, dtype=mat.dtype)
        buf[:, :rows] = mat.T
    return np.ascontiguousarray(buf).reshape(-1), ld


def unstore(buf: np.ndarray, layout: str, rows: int, cols: int, ld: int) -> np.ndarray:
    if layout == "row":
        return buf.reshape(rows, ld)[:, :cols]
    return buf.reshape(cols, ld)[:, :rows].T


def check_float(gpu: np.ndarray, ref: np.ndarray, what: str = "", tight: bool = True):
    """The two accuracy gates for floating-point results, plus the tighter arithmetic bound."""
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite output"
    err = np.abs(gpu - ref)
    worst = np.max(err / (np.abs(ref) + 1.0)) if err.size else 0.0
    assert worst <= GATE_ELEM, f"{what}: elementwise gate {worst:.3e} > {GATE_ELEM}"
    nref = np.linalg.norm(ref.reshape(-1))
    fro = np.linalg.norm((gpu - ref).reshape(-1)) / nref if nref > 0 else np.linalg.norm((gpu - ref).reshape(-1))
    assert fro <= GATE_FRO, f"{what}: Frobenius gate {fro:.3e} > {GATE_FRO}"
    if tight:
        assert fro <= TIGHT_FRO, f"{what}: relative Frobenius error {fro:.3e} above the fp32-accumulation bound"
    return worst, fro
