"""Pins of the oracle's hidden-state-to-logits step and of the two estimators applied to such logits.

What fixes the result independently of the code under test: a library matrix product in float64, a
one-hot hidden state (the logits are then one column of the weight matrix), and inputs whose
products and sums are exactly representable, for which the logits equal an integer matrix product
and every score must equal, to the last bit, what the stored-logit entry points return."""
import numpy as np

import oracle


def bf16_bits(a):
    """float32 values that are exactly representable in bf16 -> their 16-bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    assert not (bits & 0xFFFF).any(), "value is not a bf16 number"
    return (bits >> 16).astype(np.uint16)


def round_to_bf16(a):
    """Round-to-nearest-even to bf16, returned as float32."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32)


def test_lmhead_row_equals_library_matmul():
    rng = np.random.default_rng(11)
    V, d = 37, 96
    h = round_to_bf16(rng.standard_normal(d))
    W = round_to_bf16(rng.standard_normal((V, d)) * 0.05)
    x = oracle.lmhead_row(bf16_bits(h), bf16_bits(W))
    want = W.astype(np.float64) @ h.astype(np.float64)
    assert x.shape == (V,)
    assert np.abs(x - want).max() <= 1e-13 * np.abs(W.astype(np.float64)).dot(np.abs(h.astype(np.float64))).max()
    # not the transposed product, not a shifted row
    assert np.abs(x - np.roll(want, 1)).max() > 1e-3


def test_one_hot_hidden_state_selects_a_weight_column():
    rng = np.random.default_rng(12)
    V, d = 50, 64
    W = round_to_bf16(rng.standard_normal((V, d)))
    for k in (0, 17, d - 1):
        h = np.zeros(d, np.float32)
        h[k] = 1.0
        assert np.array_equal(oracle.lmhead_row(bf16_bits(h), bf16_bits(W)), W[:, k].astype(np.float64))
        h[k] = -2.0
        assert np.array_equal(oracle.lmhead_row(bf16_bits(h), bf16_bits(W)), -2.0 * W[:, k].astype(np.float64))


def test_scores_on_exact_logits_equal_the_stored_logit_entry_points():
    rng = np.random.default_rng(13)
    N, V, d = 24, 211, 48
    Hi = rng.integers(-8, 9, size=(N, d))                   # integers: exact in bf16
    Wi = rng.integers(-16, 17, size=(V, d))                 # multiples of 1/64 after scaling
    H = Hi.astype(np.float32)
    W = (Wi / 64.0).astype(np.float32)
    logits = (Hi @ Wi.T).astype(np.float64) / 64.0           # |sum| < 48*8*16 = 6144: exact in float32 too
    logits32 = logits.astype(np.float32)
    assert np.array_equal(logits32.astype(np.float64), logits)
    seeds = np.array([0x0123456789ABCDEF, 42], dtype=np.uint64)
    sid = (np.arange(N) % 2).astype(np.int32)
    pos = np.arange(N, dtype=np.uint32) * 3
    T = 0.75
    cg = rng.integers(0, V, size=N).astype(np.int32)
    ci = rng.integers(0, V, size=N).astype(np.int32)
    assert (cg != ci).any()
    g, i, x = oracle.lmhead_score(bf16_bits(H), bf16_bits(W), T, seeds, sid, pos, cg, ci, sigma=0.02, eps=1e-20,
                                  want_logits=True)
    assert np.array_equal(x, logits)
    g0 = oracle.gumbel_score(logits32, V, T, seeds, sid, pos, cg)
    i0 = oracle.ipt_score(logits32, V, T, seeds, sid, pos, ci, sigma=0.02, eps=1e-20)
    for k in g0:
        assert np.array_equal(g[k], g0[k]), k
    for k in i0:
        assert np.array_equal(i[k], i0[k]), k
    # sampling mode and per-row temperatures route through as well
    temps = np.linspace(0.5, 1.5, N).astype(np.float32)
    g, i = oracle.lmhead_score(bf16_bits(H), bf16_bits(W), T, seeds, sid, pos, None, None, temperatures=temps)
    g0 = oracle.gumbel_score(logits32, V, T, seeds, sid, pos, None, temperatures=temps)
    i0 = oracle.ipt_score(logits32, V, T, seeds, sid, pos, None, temperatures=temps)
    assert np.array_equal(g["argmax"], g0["argmax"]) and np.array_equal(i["ipt_token"], i0["ipt_token"])
    assert (g["flags"] & 2).all() and np.isnan(g["margin"]).all()
