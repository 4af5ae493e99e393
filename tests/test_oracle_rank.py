"""Pins for the oracle's logit rank and three-class classifier (Sec. 7.1, appendix algorithm
"risk classification via score and rank"): numpy / scipy ranking, and the classifier's truth table."""
import math

import numpy as np
from scipy import stats


def test_rank_matches_library_ranking(oracle_lib):
    import torch

    rng = np.random.default_rng(41)
    for V in (1, 2, 17, 1000):
        x = rng.normal(0, 2, size=V)
        x[rng.integers(0, V, size=V // 5)] = 0.5                    # ties
        if V > 5:
            x[3] = -np.inf
            x[4] = -0.0
            x[5] = 0.0
        order = stats.rankdata(-x, method="min") - 1                # 0 = highest, ties share the best rank
        for t in range(V):
            assert oracle_lib.logit_rank_row(x, t) == int((x > x[t]).sum()) == int(order[t])
        assert oracle_lib.logit_rank_row(x, -1) == -1 and oracle_lib.logit_rank_row(x, V) == -1
    # batch form on bf16 storage; rank is about raw logits: temperature does not enter
    x = torch.from_numpy(rng.normal(0, 3, size=(6, 40)).astype(np.float32)).to(torch.bfloat16)
    claimed = np.array([0, 39, 7, -1, 40, 12], dtype=np.int32)
    got = oracle_lib.logit_rank(x.view(torch.int16).numpy().view(np.uint16)[:, :], 40, claimed)
    xf = x.to(torch.float64).numpy()
    want = [int((xf[n] > xf[n, c]).sum()) if 0 <= c < 40 else -1 for n, c in enumerate(claimed)]
    assert list(got) == want


def test_classifier_truth_table(oracle_lib):
    V, R, tau = 151936, 8, 0.25
    scores = np.array([0.0, 0.25, 0.2500001, 3.0, 3.0, 3.0, np.nan, 0.1, 9.0])
    ranks = np.array([500, 500, 0, 7, 8, -1, 0, -1, 151935], dtype=np.int32)
    out = oracle_lib.classify(scores, ranks, tau, R, V)
    assert list(out["cls"]) == [0, 0, 1, 1, 2, 2, 2, 0, 2]
    want_bits = [0, 0, 3, 3, math.log2(V), math.log2(V), math.log2(V), 0, math.log2(V)]
    assert np.allclose(out["bits"], want_bits, atol=1e-12)
    # rank cutoffs of the paper's ablation: 1 -> 0 bits, 4 -> 2 bits, 8 -> 3 bits; none -> two classes only
    for R2, b in ((1, 0.0), (4, 2.0), (8, 3.0)):
        o = oracle_lib.classify(np.array([1.0]), np.array([0], dtype=np.int32), tau, R2, V)
        assert o["cls"][0] == 1 and o["bits"][0] == b
    o = oracle_lib.classify(np.array([1.0, 0.0]), np.array([0, 0], dtype=np.int32), tau, 0, V)
    assert list(o["cls"]) == [2, 0]
    # admissible-set sizes, when known, price the SAFE tokens
    o = oracle_lib.classify(np.array([0.0, 1.0]), np.array([3, 3], dtype=np.int32), tau, 8, V, np.array([1.5, 9.0]))
    assert list(o["bits"]) == [1.5, 3.0]
