"""Error measures used by the parity checks (no method arithmetic)."""
from __future__ import annotations

import numpy as np


def floored_rel_err(got, want, floor_frac=1e-3):
    """max_i |got_i - want_i| / max(|want_i|, floor_frac * max_j |want_j|).

    Element-wise relative error with the denominator floored at a small fraction of the
    tensor's largest magnitude, so that elements at a sign change do not dominate.
    """
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    scale = np.abs(want).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    den = np.maximum(np.abs(want), floor_frac * scale)
    return float((np.abs(got - want) / den).max())


def max_norm_err(got, want):
    """max|got - want| / max|want|."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    scale = np.abs(want).max()
    return float(np.abs(got - want).max() / (scale if scale > 0 else 1.0))
