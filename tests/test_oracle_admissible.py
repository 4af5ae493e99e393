"""Pins of the oracle's admissible-set count  #{ v : max_w y_w - y_v <= delta }  (Sec. 7).

Independent of the code under test: explicit sorting of scores rebuilt in Python from the raw noise
words; the special cases delta = 0 and delta = infinity; the claimed token is admissible exactly when
its margin is at most delta; and the law of the count.  For Gumbel-perturbed scores the points y_v
form (for a large vocabulary without a dominant token) a Poisson process with intensity exp(-(y - lse)),
for which the number of points within delta below the maximum, the maximum excluded, is geometric:
P(count - 1 = n) = (1 - q) q^n with q = 1 - exp(-delta), so E[count] = exp(delta)."""
import math

import numpy as np

import oracle


def _scores(x, T, seed, seq, pos):
    V = len(x)
    bits = oracle.noise_row(seed, seq, pos, 0, V)
    return np.array([x[v] / T + oracle.uniform_to_gumbel(oracle.bits_to_uniform(int(bits[v]))) for v in range(V)])


def test_count_equals_explicit_sorting():
    rng = np.random.default_rng(21)
    for V, T, delta in ((7, 1.0, 0.5), (64, 0.7, 2.0), (300, 1.3, 4.0), (300, 1.0, 0.0)):
        x = rng.standard_normal(V) * 2.0
        seed, seq, pos = 0x9E3779B97F4A7C15, 3, 11
        y = np.sort(_scores(x, T, seed, seq, pos))[::-1]
        want = int(np.sum(y[0] - y <= delta))
        c, lo, hi = oracle.admissible_count_row(x, T, seed, seq, pos, delta, tol=1e-9)
        assert c == want and lo <= c <= hi
        # the k-th largest score is admissible exactly when delta reaches its distance from the top
        for k in (1, 2, min(5, V - 1)):
            d = y[0] - y[k]
            assert oracle.admissible_count_row(x, T, seed, seq, pos, d * (1 + 1e-12))[0] >= k + 1
            assert oracle.admissible_count_row(x, T, seed, seq, pos, d * (1 - 1e-9))[0] <= k


def test_special_cases_and_monotonicity():
    rng = np.random.default_rng(22)
    V = 500
    x = rng.standard_normal(V)
    x[[3, 77]] = -np.inf                                     # masked entries are never admissible
    seed, seq, pos = 12345, 0, 9
    assert oracle.admissible_count_row(x, 1.0, seed, seq, pos, 0.0)[0] == 1
    assert oracle.admissible_count_row(x, 1.0, seed, seq, pos, 1e300)[0] == V - 2
    last = 0
    for delta in np.linspace(0, 12, 25):
        c, lo, hi = oracle.admissible_count_row(x, 1.0, seed, seq, pos, delta, tol=0.25)
        assert c >= last and lo <= c <= hi
        assert lo == oracle.admissible_count_row(x, 1.0, seed, seq, pos, delta - 0.25)[0] if delta >= 0.25 else lo <= 1
        assert hi == oracle.admissible_count_row(x, 1.0, seed, seq, pos, delta + 0.25)[0]
        last = c


def test_claimed_token_is_admissible_iff_margin_at_most_delta():
    rng = np.random.default_rng(23)
    N, V = 40, 256
    logits = (rng.standard_normal((N, V)) * 1.5).astype(np.float32)
    seeds = np.array([7, 8], dtype=np.uint64)
    sid = (np.arange(N) % 2).astype(np.int32)
    pos = np.arange(N, dtype=np.uint32)
    claims = rng.integers(0, V, size=N).astype(np.int32)
    g = oracle.gumbel_score(logits, V, 0.9, seeds, sid, pos, claims)
    delta = float(np.median(g["margin"]))
    a = oracle.admissible_count(logits, V, 0.9, seeds, sid, pos, delta)
    # removing the claimed token from the vocabulary (masking it) lowers the count by one exactly
    # when the claimed token was admissible, unless it was the maximum itself
    for n in range(N):
        if g["flags"][n] & 1:
            continue
        masked = logits[n:n + 1].copy()
        masked[0, claims[n]] = -np.inf
        b = oracle.admissible_count(masked, V, 0.9, seeds, sid[n:n + 1], pos[n:n + 1], delta)
        assert a["count"][n] - b["count"][0] == int(g["margin"][n] <= delta)


def test_count_follows_the_geometric_law():
    rng = np.random.default_rng(24)
    N, V, delta = 3000, 4096, 1.5
    logits = (rng.standard_normal((N, V))).astype(np.float32)          # no dominant token: max softmax prob ~ 1e-2
    seeds = np.array([0xABCDEF12345], dtype=np.uint64)
    sid = np.zeros(N, np.int32)
    pos = np.arange(N, dtype=np.uint32)
    c = oracle.admissible_count(logits, V, 1.0, seeds, sid, pos, delta)["count"].astype(np.float64)
    q = 1.0 - math.exp(-delta)
    mean, var = 1.0 / (1.0 - q), q / (1.0 - q) ** 2                    # of count = 1 + Geometric
    assert abs(c.mean() - mean) < 5.0 * math.sqrt(var / N) + 0.03 * mean
    assert abs((c == 1).mean() - (1.0 - q)) < 5.0 * math.sqrt(q * (1 - q) / N) + 0.01
    assert abs((c == 2).mean() - (1.0 - q) * q) < 5.0 * math.sqrt(0.25 / N) + 0.01
