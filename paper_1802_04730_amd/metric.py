"""The acceptance metric for GPU-vs-oracle parity.

err = max over elements of |gpu - ref| / (|ref| + 1e-3 * max|ref|); the bar is
2e-5.  The floor term keeps the ratio finite for outputs near zero.
"""
from __future__ import annotations

import numpy as np

PARITY_BAR = 2e-5


def parity_error(gpu, ref) -> float:
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if gpu.shape != ref.shape:
        raise ValueError("shape mismatch %s vs %s" % (gpu.shape, ref.shape))
    if ref.size == 0:
        return 0.0
    if not np.all(np.isfinite(gpu)):
        return float("inf")
    floor = 1e-3 * float(np.max(np.abs(ref)))
    den = np.abs(ref) + floor
    if floor == 0.0:
        den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(gpu - ref) / den))
