"""Pins of the oracle's Token-IPT-DiFR under the sampler's top-k / top-p filter.

Independent of the code under test: an explicit numpy implementation of the filter and of the CDF over
the kept tokens, the special case "no filter" (must reproduce the unfiltered, separately pinned function
bit for bit), the tiling property (for any u exactly one kept token matches), chi-square of the sampler's
tokens against the renormalised probabilities, and a claimed token outside the kept set."""
import numpy as np
from scipy.stats import chi2

import oracle


def explicit(x, T, k, p):
    """(kept indices in rank order, renormalised probabilities over the vocabulary)"""
    order = np.lexsort((np.arange(len(x)), -x))                   # logit descending, index ascending
    kept = order[:k] if 0 < k < len(x) else order
    if p < 1.0:
        w = np.exp((x[kept] - x[kept[0]]) / T)
        cum = np.cumsum(w / w.sum())
        kept = kept[:int(np.searchsorted(cum, p, side="left")) + 1]
    prob = np.zeros(len(x))
    w = np.exp((x[kept] - x[kept[0]]) / T)
    prob[kept] = w / w.sum()
    return kept, prob


def batch(x, T, claims, k, p, seeds=(12345,), positions=None):
    N, V = x.shape
    seeds = np.array(seeds, dtype=np.uint64)
    sid = np.zeros(N, np.int32)
    pos = np.arange(N, dtype=np.uint32) if positions is None else positions
    return oracle.ipt_filtered_score(x.astype(np.float32), V, T, seeds, sid, pos, claims, k, p), seeds, sid, pos


def test_interval_matches_explicit_filter_and_cumsum():
    rng = np.random.default_rng(31)
    N, V = 30, 97
    x = np.round(rng.standard_normal((N, V)) * 2, 1).astype(np.float32).astype(np.float64)   # coarse: ties
    claims = rng.integers(0, V, size=N).astype(np.int32)
    for k, p in ((10, 1.0), (50, 0.95), (0, 0.7), (5, 0.5), (200, 1.0)):
        r, *_ = batch(x, 0.8, claims, k, p)
        for n in range(N):
            kept, prob = explicit(x[n], 0.8, k, p)
            F = np.concatenate(([0.0], np.cumsum(prob)))
            t = claims[n]
            assert r["kept"][n] == len(kept)
            assert abs(r["cdf_lo"][n] - F[t]) < 1e-12 and abs(r["cdf_hi"][n] - F[t + 1]) < 1e-12
            u = r["u"][n]
            assert abs(r["dist"][n] - max(F[t] - u, u - F[t + 1], 0.0)) < 1e-12
            assert bool(r["flags"][n] & 1) == (F[t] <= u < F[t + 1])
            if t not in kept:
                assert r["cdf_lo"][n] == r["cdf_hi"][n] and not (r["flags"][n] & 1)
            # the sampler's token: the kept token whose interval holds u
            want = int(np.searchsorted(F[1:], u, side="right"))
            while prob[want] == 0.0:
                want += 1
            assert r["ipt_token"][n] == want and prob[r["ipt_token"][n]] > 0


def test_no_filter_is_the_unfiltered_estimator():
    rng = np.random.default_rng(32)
    N, V = 25, 300
    x = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    claims = rng.integers(0, V, size=N).astype(np.int32)
    r, seeds, sid, pos = batch(x.astype(np.float64), 1.1, claims, 0, 1.0)
    r0 = oracle.ipt_score(x, V, 1.1, seeds, sid, pos, claims)
    for key in ("u", "ipt_token", "flags"):
        assert np.array_equal(r[key], r0[key]), key
    for key in ("cdf_lo", "cdf_hi", "dist"):       # the two normalise by a different reference (top logit vs max x/T): rounding only
        assert np.abs(r[key] - r0[key]).max() < 1e-14, key
    assert (r["kept"] == V).all()


def test_filtered_sampler_follows_the_renormalised_distribution():
    rng = np.random.default_rng(33)
    V, k, p, T = 12, 6, 0.9, 1.0
    x1 = rng.standard_normal(V) * 1.5
    kept, prob = explicit(x1.astype(np.float32).astype(np.float64), T, k, p)
    N = 60000
    x = np.tile(x1, (N, 1))
    r, *_ = batch(x, T, None, k, p, positions=np.arange(N, dtype=np.uint32))
    counts = np.bincount(r["ipt_token"], minlength=V).astype(np.float64)
    assert counts[prob == 0].sum() == 0
    live = prob > 0
    stat = ((counts[live] - N * prob[live]) ** 2 / (N * prob[live])).sum()
    assert stat < chi2.ppf(1 - 1e-4, int(live.sum()) - 1), stat
    # an honest claim (the sampler's own token) always matches with distance 0
    r2, *_ = batch(x[:500], T, r["ipt_token"][:500].astype(np.int32), k, p, positions=np.arange(500, dtype=np.uint32))
    assert (r2["flags"] & 1).all() and (r2["dist"] == 0).all()


def test_signed_zeros_are_equal_logits():
    """-0 and +0 are the same logit value: between them the lower index ranks first, whatever the sign.  By hand:
    x = (0, -0, 0, -0, 1), top-3 = {4, 0, 1}; with T = 1 the kept masses are e, 1, 1."""
    x = np.array([[0.0, -0.0, 0.0, -0.0, 1.0]] * 4, dtype=np.float32)
    claims = np.array([0, 1, 2, 3], np.int32)
    out, *_ = batch(x, 1.0, claims, 3, 1.0)
    assert (out["kept"] == 3).all()
    Z = np.e + 2.0
    assert np.allclose(out["cdf_lo"], [0.0, 1 / Z, 2 / Z, 2 / Z], atol=1e-12)
    assert np.allclose(out["cdf_hi"], [1 / Z, 2 / Z, 2 / Z, 2 / Z], atol=1e-12)   # tokens 2 and 3 are outside: empty
    # the same under a nucleus: masses (e, 1, 1, 1, 1) / (e + 4), p = 0.7 needs e + 2 of them: tokens 4, 0, 1
    out, *_ = batch(x, 1.0, claims, 0, 0.7)
    assert (out["kept"] == 3).all()
    assert np.allclose(out["cdf_hi"] - out["cdf_lo"], [1 / Z, 1 / Z, 0.0, 0.0], atol=1e-12)


def test_a_marginal_token_moves_an_interval_end_by_at_most_one_over_kept():
    """The members of K are the most probable tokens, so the least probable of them - the one a cut that is in doubt adds
    or drops - holds at most 1 / |K| of the renormalised mass.  That is what the GPU comparison of the bare nucleus
    allows an interval end to move by per token in doubt (tests/test_gpu_nucleus.py); here it is checked on the oracle
    itself, between neighbouring values of top_p, on rows of ties (where the bound is attained) and on ordinary rows."""
    rng = np.random.default_rng(8)
    N, V = 12, 900
    rows = {"constant": np.full((N, V), -1.25), "coarse": np.round(rng.normal(0, 2, (N, V)) * 2) / 2,
            "normal": rng.normal(0, 2, (N, V))}
    claims = rng.integers(0, V, N).astype(np.int32)
    checked = 0
    for name, x in rows.items():
        for p in (0.3, 0.9, 0.99):
            base, *_ = batch(x, 0.9, claims, 0, p)
            for q in (p - 0.004, p + 0.004):
                other, *_ = batch(x, 0.9, claims, 0, q)
                dk = np.abs(other["kept"] - base["kept"])
                room = dk / np.minimum(other["kept"], base["kept"]) + 1e-12
                for end in ("cdf_lo", "cdf_hi"):
                    assert (np.abs(other[end] - base[end]) <= room).all(), (name, p, q, end)
                checked += int((dk > 0).sum())
    assert checked > 20      # the neighbouring cuts did differ
