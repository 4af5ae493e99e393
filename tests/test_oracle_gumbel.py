"""Pins for the oracle's Token-DiFR row: brute force in multi-precision on tiny
vocabularies, the paper's own A_{sigma,i} form, determinism under identical logits,
invariances, and the two distributional facts the Gumbel-max trick rests on
(it samples softmax(x/T) exactly; the maximum is itself Gumbel around logsumexp)."""
import math

import mpmath
import numpy as np
import pytest
from scipy import special, stats

from test_oracle_noise import _philox_bigint


def _noise_mp(seed, seq, pos, V):
    """Gumbel noise of one row in 50-digit arithmetic from the big-integer Philox."""
    mpmath.mp.dps = 50
    g = []
    for v in range(V):
        r = _philox_bigint([v >> 2, pos, seq, 0], [seed & 0xFFFFFFFF, seed >> 32])[v & 3]
        u = mpmath.mpf(2 * (r >> 9) + 1) / mpmath.mpf(2) ** 24
        g.append(-mpmath.log(-mpmath.log(u)))
    return g


@pytest.mark.parametrize("V", [2, 3, 5, 8, 13, 16])
def test_brute_force_tiny_vocab(oracle_lib, V):
    rng = np.random.default_rng(100 + V)
    for trial in range(12):
        x = rng.normal(0, 2, size=V)
        T = float(rng.choice([0.6, 0.7, 1.0, 1.3]))
        seed = int(rng.integers(0, 1 << 63))
        seq, pos = int(rng.integers(0, 100)), int(rng.integers(0, 5000))
        t = int(rng.integers(0, V))
        g = _noise_mp(seed, seq, pos, V)
        y = [mpmath.mpf(float(x[v])) / mpmath.mpf(T) + g[v] for v in range(V)]
        order = sorted(range(V), key=lambda v: (-y[v], v))       # explicit sort, lowest index first
        got = oracle_lib.gumbel_row(x, T, seed, seq, pos, t, want_scores=True)
        assert got["argmax"] == order[0]
        assert abs(mpmath.mpf(got["max_score"]) - y[order[0]]) < 1e-12
        assert abs(mpmath.mpf(got["margin"]) - (y[order[0]] - y[t])) < 1e-12
        assert abs(mpmath.mpf(got["claimed_score"]) - y[t]) < 1e-12
        assert abs(mpmath.mpf(got["gap2"]) - (y[order[0]] - y[order[1]])) < 1e-12
        assert bool(got["flags"] & 1) == (order[0] == t)
        for v in range(V):
            assert abs(mpmath.mpf(float(got["y"][v])) - y[v]) < 1e-12


def test_margin_is_minus_min_A_over_T(oracle_lib):
    # appendix algorithm: A_i = l_t - l_i + T (G_t - G_i); the margin is -min_i A_i / T
    rng = np.random.default_rng(7)
    V = 40
    for trial in range(20):
        ell = rng.normal(0, 3, size=V)
        T = float(rng.choice([0.5, 0.8, 1.0, 2.0]))
        seed, seq, pos, t = int(rng.integers(0, 1 << 63)), 3, trial, int(rng.integers(0, V))
        bits = oracle_lib.noise_row(seed, seq, pos, 0, V)
        u = (2.0 * (bits >> np.uint32(9)).astype(np.float64) + 1.0) * 2.0 ** -24
        G = -np.log(-np.log(u))
        A = ell[t] - ell + T * (G[t] - G)
        got = oracle_lib.gumbel_row(ell, T, seed, seq, pos, t)
        assert abs(-T * got["margin"] - A.min()) < 1e-9
        assert got["argmax"] == int(np.argmin(A))


def test_honest_claim_under_identical_logits_has_zero_margin(oracle_lib):
    # the sampler is deterministic once p and the seed are fixed (Sec. 3.2)
    rng = np.random.default_rng(8)
    V = 257
    for trial in range(50):
        x = rng.normal(0, 2, size=V)
        seed = int(rng.integers(0, 1 << 63))
        sample = oracle_lib.gumbel_row(x, 0.9, seed, 1, trial, -1)
        assert sample["flags"] & 2 and math.isnan(sample["margin"])
        again = oracle_lib.gumbel_row(x, 0.9, seed, 1, trial, sample["argmax"])
        assert again["margin"] == 0.0 and again["flags"] & 1
        other = (sample["argmax"] + 1) % V
        wrong = oracle_lib.gumbel_row(x, 0.9, seed, 1, trial, other)
        assert wrong["margin"] > 0.0 and not wrong["flags"] & 1
        assert wrong["margin"] >= wrong["gap2"] > 0


def test_invariances_and_dominant_logit(oracle_lib):
    rng = np.random.default_rng(9)
    V = 100
    for trial in range(20):
        x = rng.normal(0, 2, size=V)
        seed, t = int(rng.integers(0, 1 << 63)), int(rng.integers(0, V))
        base = oracle_lib.gumbel_row(x, 0.7, seed, 2, trial, t)
        assert base["margin"] >= 0
        shifted = oracle_lib.gumbel_row(x + 3.25, 0.7, seed, 2, trial, t)          # x + c
        assert shifted["argmax"] == base["argmax"] and abs(shifted["margin"] - base["margin"]) < 1e-11
        assert abs(shifted["max_score"] - base["max_score"] - 3.25 / 0.7) < 1e-11
        scaled = oracle_lib.gumbel_row(x * 2.0, 1.4, seed, 2, trial, t)            # (x a, T a)
        assert scaled["argmax"] == base["argmax"] and abs(scaled["margin"] - base["margin"]) < 1e-11
        # different position or sequence or seed -> different noise
        assert oracle_lib.gumbel_row(x, 0.7, seed, 2, trial + 1, t)["max_score"] != base["max_score"]
        assert oracle_lib.gumbel_row(x, 0.7, seed, 3, trial, t)["max_score"] != base["max_score"]
        # one logit far above the rest always wins
        xd = x.copy()
        j = int(rng.integers(0, V))
        xd[j] += 50.0
        assert oracle_lib.gumbel_row(xd, 0.7, seed, 2, trial, t)["argmax"] == j
        # -inf entries are masked: never the argmax
        xm = x.copy()
        xm[base["argmax"]] = -np.inf
        assert oracle_lib.gumbel_row(xm, 0.7, seed, 2, trial, t)["argmax"] != base["argmax"]


def test_ties_go_to_lowest_index(oracle_lib):
    # equal noise cannot be forced, but equal scores can: with all logits -inf except
    # duplicates of a huge value the noise still separates them; instead check via y:
    x = np.zeros(8)
    out = oracle_lib.gumbel_row(x, 1.0, 5, 0, 0, 0, want_scores=True)
    y = out["y"]
    assert out["argmax"] == int(np.argmax(y))                 # numpy argmax = first maximum
    # a constructed exact tie: masked row where every finite entry is -inf gives y = -inf everywhere
    out = oracle_lib.gumbel_row(np.full(8, -np.inf), 1.0, 5, 0, 0, 3)
    assert out["argmax"] == 0


def test_batch_matches_row_and_nonfinite_flag(oracle_lib):
    import torch

    rng = np.random.default_rng(10)
    N, V, ld = 9, 50, 56
    x = torch.from_numpy(rng.normal(0, 2, size=(N, ld)).astype(np.float32)).to(torch.bfloat16)
    xb = x.view(torch.int16).numpy().view(np.uint16)
    seeds = np.array([11, 22, 33], dtype=np.uint64)
    seq_ids = np.array([0, 0, 0, 1, 1, 1, 2, 2, 2], dtype=np.int32)
    positions = np.array([0, 1, 2, 0, 1, 2, 0, 1, 2], dtype=np.uint32)
    claimed = rng.integers(0, V, size=N).astype(np.int32)
    claimed[4] = V            # out of range
    temps = np.linspace(0.5, 1.5, N).astype(np.float32)
    out = oracle_lib.gumbel_score(xb, V, 1.0, seeds, seq_ids, positions, claimed, temps)
    for n in range(N):
        row = oracle_lib.gumbel_row(x[n, :V].to(torch.float64).numpy(), float(temps[n]), int(seeds[seq_ids[n]]),
                                    int(seq_ids[n]), int(positions[n]), int(claimed[n]))
        for k in ("margin", "max_score", "claimed_score", "gap2"):
            assert (out[k][n] == row[k]) or (math.isnan(out[k][n]) and math.isnan(row[k]))
        assert out["argmax"][n] == row["argmax"] and out["flags"][n] == row["flags"]
    assert out["flags"][4] & 2 and math.isnan(out["margin"][4])
    xf = rng.normal(0, 1, size=(2, 16)).astype(np.float32)
    xf[1, 5] = np.nan
    o2 = oracle_lib.gumbel_score(xf, 16, 1.0, seeds, np.zeros(2, np.int32), np.arange(2, dtype=np.uint32))
    assert not o2["flags"][0] & 4 and o2["flags"][1] & 4
    assert (o2["flags"] & 2).all()                           # claimed=None -> sampling mode


def test_sample_frequencies_match_softmax(oracle_lib):
    # Gumbel-max is an exact sampler of softmax(x/T) (Sec. 3.2): chi-square over (seed, position) pairs
    V, T = 12, 0.8
    rng = np.random.default_rng(11)
    x = rng.normal(0, 1.5, size=V).astype(np.float32)
    S, L = 500, 400
    logits = np.broadcast_to(x, (S * L, V)).copy()
    seeds = rng.integers(0, 1 << 63, size=S).astype(np.uint64)
    seq_ids = np.repeat(np.arange(S, dtype=np.int32), L)
    positions = np.tile(np.arange(L, dtype=np.uint32), S)
    out = oracle_lib.gumbel_score(logits, V, T, seeds, seq_ids, positions)
    counts = np.bincount(out["argmax"], minlength=V)
    p = special.softmax(x.astype(np.float64) / T)
    chi = stats.chisquare(counts, p * counts.sum())
    assert chi.pvalue > 1e-4, (counts, p)
    # and it is not, e.g., softmax(x) at the wrong temperature or of -x
    assert stats.chisquare(counts, special.softmax(x.astype(np.float64)) * counts.sum()).pvalue < 1e-6


def test_max_is_gumbel_around_logsumexp(oracle_lib):
    # max_v (x_v/T + g_v) - logsumexp(x/T) ~ Gumbel(0,1)
    V, T = 64, 0.7
    rng = np.random.default_rng(12)
    N = 20000
    logits = rng.normal(0, 2, size=(N, V)).astype(np.float32)
    seeds = rng.integers(0, 1 << 63, size=50).astype(np.uint64)
    seq_ids = (np.arange(N) % 50).astype(np.int32)
    positions = (np.arange(N) // 50).astype(np.uint32)
    out = oracle_lib.gumbel_score(logits, V, T, seeds, seq_ids, positions)
    z = out["max_score"] - special.logsumexp(logits.astype(np.float64) / T, axis=1)
    assert stats.kstest(z, "gumbel_r").pvalue > 1e-4
