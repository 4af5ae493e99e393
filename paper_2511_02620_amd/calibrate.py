"""Host-side threshold calibration on benign pooled scores.

The paper calibrates the flagging threshold on benign traffic to a target false-positive
rate (Sec. 5.2; appendix on score statistics: pick the percentile of the benign score
distribution).  Scores here are suspiciousness (larger = more suspicious), so the
threshold is the ceil((1 - fpr) n)-th smallest benign value: at most floor(fpr n) benign
units lie strictly above it.  The result is rounded up to fp32 because the library's
threshold argument is a float.
"""
from __future__ import annotations

import math

import numpy as np


def threshold_for_fpr(benign_scores, fpr: float) -> float:
    m = np.sort(np.asarray(benign_scores, dtype=np.float64).ravel())
    n = m.shape[0]
    if n == 0:
        raise ValueError("no benign scores to calibrate on")
    if not (0.0 <= fpr < 1.0):
        raise ValueError("fpr must be in [0, 1)")
    k = min(max(int(math.ceil((1.0 - fpr) * n)), 1), n)
    tau = float(m[k - 1])
    t32 = np.float32(tau)
    if float(t32) < tau:
        t32 = np.nextafter(t32, np.float32(np.inf))
    return float(t32)
