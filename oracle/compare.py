"""Error metrics used when a result is held against the oracle.  TEST INFRASTRUCTURE ONLY (no loss arithmetic here).

Tolerances follow the stated targets: fp32 path 1e-5, bf16 path 2e-2, measured as
  - loss / lse: per position, |x - ref| / max(|loss_ref|, |lse_ref|, 1e-6)   (loss is a difference of lse and o+,
    so its rounding error scales with those, not with the possibly tiny loss itself);
  - dH, dE: per tensor, max|x - ref| / max|ref|  (dE over the rows the oracle touched);
  - dH, dE, per row (row_rel): every row against its OWN largest entry, max_t|x[r,t] - ref[r,t]| / max(max_t|ref[r,t]|,
    floor), floor = floor_frac * max|ref| of the whole tensor.  With power-law targets the largest dE rows are those of
    a few hot correct items (thousands of summed terms); the per-tensor metric alone would let a negative's row, whose
    entries are a thousandth of that, be entirely wrong.  The floor keeps rows that are zero up to cancellation
    (their error is absolute, set by the terms that cancelled) from dividing by nothing.
Masked positions and untouched dE rows are compared exactly by the callers.
"""
from __future__ import annotations

import numpy as np


def per_position_rel(x, ref_loss, ref_lse, ref) -> float:
    x = np.asarray(x, np.float64)
    den = np.maximum(np.maximum(np.abs(ref_loss), np.abs(ref_lse)), 1e-6)
    if x.size == 0:
        return 0.0
    return float(np.max(np.abs(x - ref) / den))


def tensor_rel(x, ref) -> float:
    x = np.asarray(x, np.float64)
    if x.size == 0:
        return 0.0
    den = max(float(np.max(np.abs(ref))), 1e-30)
    return float(np.max(np.abs(x - ref))) / den


def row_rel(x, ref, floor_frac: float = 1e-3) -> float:
    """Largest per-row error, each row relative to its own max-norm (not below floor_frac * the tensor's max-norm)."""
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    if x.size == 0:
        return 0.0
    x = x.reshape(-1, x.shape[-1])
    ref = ref.reshape(-1, ref.shape[-1])
    floor = floor_frac * max(float(np.max(np.abs(ref))), 1e-30)
    den = np.maximum(np.max(np.abs(ref), axis=1), floor)
    return float(np.max(np.max(np.abs(x - ref), axis=1) / den))
