"""Shared pieces of the GPU parity tests: device marshalling, gates, call wrappers."""
from __future__ import annotations

import numpy as np

from paper_2505_02146_amd.gates import GATE_ELEM, GATE_FRO, TIGHT_FRO, check_float  # noqa: F401  (re-exported)


def dev(a: np.ndarray, bf16: bool = False):
    """numpy host array -> torch tensor on cuda:0 (uint16 bf16 bits travel as int16)."""
    from paper_2505_02146_amd import xp
    return xp.to_device(a)


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
