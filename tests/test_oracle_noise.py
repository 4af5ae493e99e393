"""Pins for the oracle's noise path: Philox4x32-10 and the bits -> uniform -> Gumbel map.

None of these re-use the oracle's own code: known-answer vectors, a structurally
different big-integer Philox, closed forms, moments and a KS test.
"""
import math
import os

import mpmath
import numpy as np
import pytest
from scipy import stats

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_lines():
    out = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        out.append(line.split())
    return out


def test_philox_known_answers(oracle_lib):
    lines = _kat_lines()
    assert len(lines) == 3
    pinned = 0
    for toks in lines:
        ctr = [int(t, 16) for t in toks[0:4]]
        key = [int(t, 16) for t in toks[4:6]]
        got = oracle_lib.philox4x32_10(ctr, key)
        for j, t in enumerate(toks[6:10]):
            if set(t) == {"-"}:
                continue
            assert int(got[j]) == int(t, 16), (toks, j, hex(int(got[j])))
            pinned += 1
    assert pinned >= 11


def _philox_bigint(ctr, key):
    """Philox4x32-10 written with Python integers and divmod (no fixed-width types):
    the multiply is an exact big product split by divmod(., 2**32)."""
    B = 1 << 32
    c = list(ctr)
    k = list(key)
    for rnd in range(10):
        hi0, lo0 = divmod(0xD2511F53 * c[0], B)
        hi1, lo1 = divmod(0xCD9E8D57 * c[2], B)
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + 0x9E3779B9) % B, (k[1] + 0xBB67AE85) % B]
    return c


def test_philox_bigint_reproduces_kats():
    # the independent implementation itself reproduces the published vectors
    for toks in _kat_lines():
        got = _philox_bigint([int(t, 16) for t in toks[0:4]], [int(t, 16) for t in toks[4:6]])
        for j, t in enumerate(toks[6:10]):
            if set(t) != {"-"}:
                assert got[j] == int(t, 16)


def test_philox_matches_bigint_on_random_inputs(oracle_lib):
    rng = np.random.default_rng(20251102)
    for _ in range(2000):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, size=4, dtype=np.uint64)]
        key = [int(x) for x in rng.integers(0, 1 << 32, size=2, dtype=np.uint64)]
        assert [int(x) for x in oracle_lib.philox4x32_10(ctr, key)] == _philox_bigint(ctr, key)


def test_philox_is_injective_on_counters(oracle_lib):
    # a keyed Philox block is a bijection of the 128-bit counter
    key = [0x12345678, 0x9ABCDEF0]
    seen = set()
    for c0 in range(1 << 12):
        out = tuple(int(x) for x in oracle_lib.philox4x32_10([c0, 7, 3, 0], key))
        seen.add(out)
    assert len(seen) == 1 << 12


def test_noise_word_counter_layout(oracle_lib):
    # noise word v of (seed, seq, pos, stream) = output word v&3 of the block with
    # counter (v>>2, pos, seq, stream) and key (seed low, seed high)
    seed = 0xDEADBEEFCAFEF00D
    for v in [0, 1, 2, 3, 4, 5, 1023, 151935, (1 << 33) + 6]:
        for stream in (0, 1):
            blk = _philox_bigint([(v >> 2) & 0xFFFFFFFF, 77, 5, stream], [seed & 0xFFFFFFFF, seed >> 32])
            assert oracle_lib.noise_word(seed, 5, 77, stream, v) == blk[v & 3]
    row = oracle_lib.noise_row(seed, 5, 77, 0, 37)
    assert [int(x) for x in row] == [oracle_lib.noise_word(seed, 5, 77, 0, v) for v in range(37)]


def test_noise_bits_avalanche(oracle_lib):
    # flipping one input bit flips about half of the output bits
    seed = 0x0123456789ABCDEF
    base = oracle_lib.noise_row(seed, 1, 9, 0, 4096)
    for other in (oracle_lib.noise_row(seed ^ 1, 1, 9, 0, 4096), oracle_lib.noise_row(seed, 1, 8, 0, 4096),
                  oracle_lib.noise_row(seed, 0, 9, 0, 4096), oracle_lib.noise_row(seed, 1, 9, 1, 4096)):
        flipped = np.unpackbits((base ^ other).view(np.uint8)).mean()
        assert 0.49 < flipped < 0.51


def test_uniform_closed_forms(oracle_lib):
    o = oracle_lib
    assert o.bits_to_uniform(0) == 2.0 ** -24
    assert o.bits_to_uniform(0x1FF) == 2.0 ** -24            # low 9 bits unused
    assert o.bits_to_uniform(0x200) == 3 * 2.0 ** -24
    assert o.bits_to_uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert o.bits_to_uniform(1 << 31) == 0.5 + 2.0 ** -24
    # exactly representable in single precision, symmetric about 1/2
    rng = np.random.default_rng(1)
    for r in rng.integers(0, 1 << 32, size=2000, dtype=np.uint64):
        u = o.bits_to_uniform(int(r))
        assert 0.0 < u < 1.0
        assert float(np.float32(u)) == u
        assert o.bits_to_uniform(int(r) ^ 0xFFFFFFFF) == 1.0 - u


def test_gumbel_closed_forms_multiprecision(oracle_lib):
    o = oracle_lib
    mpmath.mp.dps = 50
    assert abs(o.uniform_to_gumbel(2.0 ** -24) - (-math.log(24 * math.log(2)))) < 1e-14
    ks = [0, 1, 2, 1000, (1 << 22) - 1, 1 << 22, (1 << 22) + 1, (1 << 23) - 1000, (1 << 23) - 2, (1 << 23) - 1]
    rng = np.random.default_rng(2)
    ks += [int(k) for k in rng.integers(0, 1 << 23, size=300)]
    for k in ks:
        u = mpmath.mpf(2 * k + 1) / mpmath.mpf(2) ** 24
        want = -mpmath.log(-mpmath.log(u))
        got = o.uniform_to_gumbel(o.bits_to_uniform(k << 9))
        assert abs(mpmath.mpf(got) - want) <= mpmath.mpf(4e-15) * max(1, abs(want)), k
    top = o.uniform_to_gumbel(o.bits_to_uniform(0xFFFFFFFF))
    assert abs(top - 16.635532) < 1e-5
    assert abs(o.uniform_to_gumbel(0.5 + 2.0 ** -24) - (-math.log(math.log(2)))) < 1e-6


def test_gumbel_moments_and_uniform_ks(oracle_lib):
    o = oracle_lib
    n = 1 << 20
    bits = np.concatenate([o.noise_row(0xABCDEF12345 + s, s, 3, 0, n // 4) for s in range(4)])
    k = (bits >> np.uint32(9)).astype(np.float64)
    u = (2 * k + 1) * 2.0 ** -24
    assert stats.kstest(u, "uniform").pvalue > 1e-4
    sample = bits[:: n // 4096][:4096]
    g_oracle = np.array([o.uniform_to_gumbel(o.bits_to_uniform(int(r))) for r in sample])
    g_numpy = -np.log(-np.log(u[:: n // 4096][:4096]))
    assert np.max(np.abs(g_oracle - g_numpy)) < 1e-7          # library logs agree away from cancellation
    g = -np.log(-np.log(u))
    # Gumbel(0,1): mean = Euler-Mascheroni, variance = pi^2/6; 5-sigma bands
    sd = math.pi / math.sqrt(6.0)
    assert abs(g.mean() - 0.5772156649) < 5 * sd / math.sqrt(n)
    var_sd = math.sqrt((5.4 - 1.0) / n) * sd * sd              # kurtosis of Gumbel = 5.4
    assert abs(g.var() - math.pi ** 2 / 6) < 5 * var_sd


def test_decode_row_exact(oracle_lib):
    import torch

    t = torch.tensor([0.0, -0.0, 1.0, -2.5, 3.140625, 1e-3, -65504.0, float("-inf"), 1.17e-38], dtype=torch.float32)
    b = t.to(torch.bfloat16)
    got = oracle_lib.decode_row(b.view(torch.int16).numpy().view(np.uint16))
    want = b.to(torch.float64).numpy()
    assert np.array_equal(got, want)
    f = np.array([1.5, -7.25, 3.0e-40, 16777217.0], dtype=np.float32)
    assert np.array_equal(oracle_lib.decode_row(f), f.astype(np.float64))
