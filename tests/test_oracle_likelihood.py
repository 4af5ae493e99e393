"""Pins of the oracle's Token-DiFR likelihood estimate (appendix algorithm of the Gumbel-max FSSL estimator).

What fixes the result independently of the code under test: closed forms (no competitor: a normal tail
probability; one competitor: Phi(A / (sigma sqrt 2))), a direct simulation of the noisy race the formula
describes (Gaussian noise on every logit, fixed filter threshold, the claimed token must survive the filter
and beat every surviving competitor), explicit Python sorting for the active set, an explicit numpy
top-k / top-p filter for the threshold, and the limits sigma -> 0."""
import math

import numpy as np
from scipy.stats import norm

import oracle


def stratified_normal(M):
    """M standard normal 'draws' that integrate smooth functions to O(1/M): quantile midpoints."""
    return norm.ppf((np.arange(M) + 0.5) / M)


def gumbel_noise(V, seed, seq, pos):
    bits = oracle.noise_row(seed, seq, pos, 0, V)
    return np.array([oracle.uniform_to_gumbel(oracle.bits_to_uniform(int(b))) for b in bits])


def explicit_tau(x, T, k, p):
    order = np.argsort(-x, kind="stable")
    kept = order[:k] if 0 < k < len(x) else order
    if p < 1.0:
        w = np.exp((x[kept] - x[kept[0]]) / T)
        cum = np.cumsum(w / w.sum())
        kept = kept[:int(np.searchsorted(cum, p, side="left")) + 1]
    return x[kept[-1]] if (k > 0 or p < 1.0) else -np.inf


ROW = dict(seeds=np.array([0x5DEECE66D1234567], dtype=np.uint64), seq_ids=np.zeros(1, np.int32),
           positions=np.array([17], dtype=np.uint32))


def one(x, T, t, k, p, s, sigma, z):
    r = oracle.likelihood(np.asarray(x, dtype=np.float32)[None, :], len(x), T, ROW["seeds"], ROW["seq_ids"],
                          ROW["positions"], np.array([t], np.int32), k, p, s, sigma, z)
    return {key: v[0] for key, v in r.items()}


def test_no_competitor_is_a_normal_tail():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(40) * 2).astype(np.float32).astype(np.float64)
    z = stratified_normal(4000)
    assert one(x, 1.0, 5, 0, 1.0, 0, 0.3, z)["pi"] == 1.0                       # no filter, nobody to lose to
    for t in (int(np.argsort(-x)[2]), int(np.argsort(-x)[7])):
        r = one(x, 1.0, t, 5, 1.0, 0, 0.7, z)                                   # top-5 filter only
        tau = np.sort(x)[-5]
        assert r["tau"] == tau
        assert abs(r["pi"] - norm.cdf((x[t] - tau) / 0.7)) < 1.0 / 4000 + 1e-12
    assert math.isnan(one(x, 1.0, -1, 5, 1.0, 0, 0.7, z)["pi"]) and math.isnan(one(x, 1.0, 40, 0, 1.0, 3, 0.7, z)["pi"])


def test_one_competitor_closed_form():
    rng = np.random.default_rng(2)
    V, T, sigma = 30, 0.8, 0.5
    x = (rng.standard_normal(V) * 1.5).astype(np.float32).astype(np.float64)
    g = gumbel_noise(V, int(ROW["seeds"][0]), 0, 17)
    y = x + T * g
    z = stratified_normal(20000)
    for t in (int(np.argmax(y)), int(np.argsort(-y)[1]), int(np.argsort(-y)[4])):
        r = one(x, T, t, 0, 1.0, 1, sigma, z)
        i = int(np.argsort(-np.where(np.arange(V) == t, -np.inf, y))[0])
        assert r["active"][0] == i
        A = x[t] - x[i] + T * (g[t] - g[i])
        # E_x Phi((x + A)/sigma), x ~ N(0, sigma^2)  =  Phi(A / (sigma sqrt 2))
        assert abs(r["pi"] - norm.cdf(A / (sigma * math.sqrt(2)))) < 2e-4
        assert abs(r["log_pi"] - math.log(r["pi"])) < 1e-12


def test_active_set_and_threshold_match_explicit_sorting():
    rng = np.random.default_rng(3)
    V, T = 200, 1.3
    x = np.round(rng.standard_normal(V) * 2, 1).astype(np.float32).astype(np.float64)     # coarse values: ties in x
    g = gumbel_noise(V, int(ROW["seeds"][0]), 0, 17)
    z = stratified_normal(64)
    for t, k, p, s in ((3, 50, 0.95, 8), (10, 7, 1.0, 16), (11, 0, 0.5, 5), (12, 20, 0.3, 1), (13, 0, 1.0, 199), (14, 0, 1.0, 400)):
        r = one(x, T, t, k, p, s, 0.4, z)
        y = np.where(np.arange(V) == t, -np.inf, x + T * g)
        want = np.argsort(-y, kind="stable")[:min(s, V - 1)]
        assert np.array_equal(r["active"][:len(want)], want) and (r["active"][len(want):] == -1).all()
        assert r["tau"] == explicit_tau(x, T, k, p)
        if 0 < s < V - 1:
            ys = np.sort(y)[::-1]
            assert abs(r["gap_s"] - (ys[s - 1] - ys[s]) / T) < 1e-12


def test_simulated_race_agrees():
    """Gaussian noise on every logit; the filter threshold stays where the verifier computed it; the claimed
    token is the sample iff it survives the filter and no surviving competitor has a larger perturbed score."""
    rng = np.random.default_rng(4)
    V, T, sigma, k = 6, 1.0, 0.8, 3
    x = np.array([1.2, 0.9, 1.0, -0.5, 0.7, 0.2])
    g = gumbel_noise(V, int(ROW["seeds"][0]), 0, 17)
    z = stratified_normal(20000)
    trials = 400000
    eps = rng.standard_normal((trials, V)) * sigma
    tau = np.sort(x)[-k]
    for t in range(V):
        r = one(x, T, t, k, 1.0, V - 1, sigma, z)
        score = x + eps + T * g
        alive = x + eps >= tau
        others = np.arange(V) != t
        beaten = np.all(~(alive[:, others] & (score[:, others] > score[:, [t]])), axis=1)
        freq = np.mean((x[t] + eps[:, t] > tau) & beaten)
        assert abs(freq - r["pi"]) < 5.0 * math.sqrt(max(freq * (1 - freq), 1e-4) / trials) + 3e-4, (t, freq, r["pi"])


def test_small_sigma_limits():
    rng = np.random.default_rng(5)
    V, T = 64, 1.0
    x = (rng.standard_normal(V) * 2).astype(np.float32).astype(np.float64)
    g = gumbel_noise(V, int(ROW["seeds"][0]), 0, 17)
    y = x + T * g
    z = stratified_normal(256)
    best, second = int(np.argsort(-y)[0]), int(np.argsort(-y)[1])
    inside = x[best] >= np.sort(x)[-10]
    r = one(x, T, best, 10, 1.0, 8, 1e-4, z)
    assert r["pi"] == (1.0 if inside else 0.0)
    assert one(x, T, second, 0, 1.0, 8, 1e-4, z)["pi"] == 0.0 and one(x, T, second, 0, 1.0, 8, 1e-4, z)["log_pi"] == -np.inf
