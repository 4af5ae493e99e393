"""The product's host-side threshold calibration against the oracle's and against its definition."""
import math

import numpy as np
import pytest

from paper_2511_02620_amd import calibrate


def test_threshold_matches_oracle_and_definition(oracle_lib):
    rng = np.random.default_rng(5)
    for n, fpr in [(253, 1e-2), (64, 1e-2), (1000, 1e-3), (50, 0.1), (9, 0.34), (1, 0.0)]:
        scores = rng.gamma(2.0, 0.01, size=n)
        tau = calibrate.threshold_for_fpr(scores, fpr)
        assert tau == oracle_lib.calibrate_threshold(scores, fpr)
        assert float(np.float32(tau)) == tau
        assert int((scores > tau).sum()) == math.floor(fpr * n + 1e-9)
    with pytest.raises(ValueError):
        calibrate.threshold_for_fpr([], 0.01)
    with pytest.raises(ValueError):
        calibrate.threshold_for_fpr([1.0], 1.0)
