"""Error figures used to compare a computed Y with the oracle's fp64 Y.  TEST INFRASTRUCTURE.

The pass/fail figure is  max_{m,n} |y - Y| / max(|Y[m,n]|, rms_n(Y[m,:]))  -- an
element-wise relative error whose denominator is floored at the row's rms, because a pure
element-wise ratio is meaningless where the sum cancels to ~0.
"""
from __future__ import annotations

import numpy as np


def parity_errors(y, Y) -> dict:
    y = np.asarray(y, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    if y.shape != Y.shape:
        raise ValueError("shape mismatch")
    if Y.size == 0:
        return {"max_rel_floored": 0.0, "max_rel_large": 0.0, "max_abs": 0.0}
    rms = np.sqrt(np.mean(Y * Y, axis=-1, keepdims=True))
    den = np.maximum(np.abs(Y), rms)
    den = np.where(den == 0.0, 1.0, den)
    diff = np.abs(y - Y)
    large = np.abs(Y) >= rms
    rel_large = float(np.max(diff[large] / np.abs(Y[large]))) if np.any(large & (Y != 0)) else 0.0
    return {
        "max_rel_floored": float(np.max(diff / den)),
        "max_rel_large": rel_large,
        "max_abs": float(np.max(diff)),
    }
