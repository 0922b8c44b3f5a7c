"""Error metrics used when a result is held against the oracle.  TEST INFRASTRUCTURE ONLY (no loss arithmetic here).

Tolerances follow the stated targets: fp32 path 1e-5, bf16 path 2e-2, measured as
  - loss / lse: per position, |x - ref| / max(|loss_ref|, |lse_ref|, 1e-6)   (loss is a difference of lse and o+,
    so its rounding error scales with those, not with the possibly tiny loss itself);
  - dH, dE: per tensor, max|x - ref| / max|ref|  (dE over the rows the oracle touched).
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
