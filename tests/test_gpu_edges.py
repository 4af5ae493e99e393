"""Degenerate shapes and extreme parameters through every row entry point, against the oracle:
vocabularies smaller than one 16-byte vector, a single row, padding columns full of garbage,
temperatures at both ends of what fp32 carries sensibly, positions / sequence ids / seeds at the ends
of their integer ranges."""
import numpy as np
import pytest
import torch

import oracle
import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def difr():
    import paper_2511_02620_amd as m
    m.load_library()
    return m


def _run_all(difr, logits, V, T, seeds, sid, pos, cg, ci, temps=None, tie_rel=parity.TIE_REL):
    host = parity.to_host_logits(logits)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    ht = None if temps is None else temps.cpu().numpy()
    g = difr.gumbel_score(logits, T, seeds, sid, pos, cg, V=V, temperatures=temps)
    i = difr.ipt_score(logits, T, seeds, sid, pos, ci, V=V, temperatures=temps, want_token=True)
    og = oracle.gumbel_score(host, V, np.float32(T), hs, hsid, hpos, cg.cpu().numpy(), ht)
    oi = oracle.ipt_score(host, V, np.float32(T), hs, hsid, hpos, ci.cpu().numpy(), ht)
    sg = parity.compare_gumbel(g, og, tie_rel=tie_rel)
    si = parity.compare_ipt(i, oi, host, V, (np.float32(T) if ht is None else ht, hs, hsid, hpos), tie_rel=tie_rel)
    aligned = logits.data_ptr() % 16 == 0 and (logits.stride(0) * logits.element_size()) % 16 == 0
    fg, fi = difr.score_both(logits, T, seeds, sid, pos, cg, ci, V=V, temperatures=temps)
    torch.cuda.synchronize()
    for k in fg:
        assert torch.equal(torch.nan_to_num(fg[k].float(), nan=-7.0), torch.nan_to_num(g[k].float(), nan=-7.0)), k
    for k in fi:
        ref = i[k] & 0xF7 if k == "flags" else i[k]          # the honest-token search above sets the SLOW_PATH bit
        assert torch.equal(torch.nan_to_num(fi[k].float(), nan=-7.0), torch.nan_to_num(ref.float(), nan=-7.0)), k
    a = difr.admissible_count(logits, T, seeds, sid, pos, g["max_score"], 1.5, V=V, temperatures=temps)
    oa = oracle.admissible_count(host, V, np.float32(T), hs, hsid, hpos, 1.5, tol=2e-5 * max(1.0, 1.0 / T), temperatures=ht)
    c = a["count"].cpu().numpy()
    assert (c >= oa["count_lo"]).all() and (c <= oa["count_hi"]).all()
    return sg, si, aligned


@pytest.mark.parametrize("dtype,V,ld", [(torch.bfloat16, 1, 8), (torch.bfloat16, 2, 8), (torch.bfloat16, 7, 8),
                                        (torch.bfloat16, 8, 8), (torch.bfloat16, 9, 16), (torch.float32, 1, 4),
                                        (torch.float32, 3, 4), (torch.float32, 5, 8), (torch.bfloat16, 3, 3),
                                        (torch.float32, 1, 1)])
def test_tiny_vocabularies_and_garbage_padding(difr, dtype, V, ld):
    N = 33
    g = torch.Generator().manual_seed(V * 100 + ld)
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)       # padding columns: NaN
    if ld > V:
        logits[::2, V:] = float("inf")                                        # ... or +inf
    logits[:, :V] = (torch.randn(N, V, generator=g) * 3).to(dtype).to(DEV)
    seeds = torch.tensor([3, 1 << 62], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    cg = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    ci = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    sg, si, _ = _run_all(difr, logits, V, 0.9, seeds, sid, pos, cg, ci)
    fl = difr.gumbel_score(logits, 0.9, seeds, sid, pos, cg, V=V)["flags"]
    assert not (fl & 4).any()                                                  # the padding was never looked at
    if V == 1:
        out = difr.gumbel_score(logits, 0.9, seeds, sid, pos, cg, V=V)
        assert (out["margin"] == 0).all() and (out["argmax"] == 0).all()
        assert (difr.ipt_score(logits, 0.9, seeds, sid, pos, ci, V=V)["dist"] == 0).all()


def test_single_row_and_integer_range_ends(difr):
    V = 4104
    g = torch.Generator().manual_seed(8)
    for N in (1, 3):
        logits = (torch.randn(N, V, generator=g) * 2).to(torch.bfloat16).to(DEV)
        seeds = torch.tensor([-1, 0, -(1 << 63)], dtype=torch.int64).to(DEV)          # 2^64-1, 0, 2^63
        sid = torch.tensor([2, 0, 1][:N], dtype=torch.int32).to(DEV)
        pos = torch.tensor([-1, 0, -(1 << 31)][:N], dtype=torch.int32).to(DEV)      # 2^32-1, 0, 2^31 as uint32
        cg = torch.tensor([V - 1, 0, 17][:N], dtype=torch.int32).to(DEV)
        ci = torch.tensor([0, V - 1, 4000][:N], dtype=torch.int32).to(DEV)
        _run_all(difr, logits, V, 1.0, seeds, sid, pos, cg, ci)


@pytest.mark.parametrize("T", [0.02, 0.1, 10.0, 300.0])
def test_extreme_temperatures(difr, T):
    """Very cold: the scores are dominated by x / T (hundreds), an fp32 ulp of a score is ~3e-5, the softmax is
    one-hot.  Very hot: the logits hardly matter.  Tolerances stay absolute 1e-4 on CDF values; margins are
    compared at 1e-4 relative to the score scale (the oracle's near-tie rule already scales that way)."""
    N, V = 40, 8200
    g = torch.Generator().manual_seed(int(T * 1000))
    logits = (torch.randn(N, V, generator=g) * 2).to(torch.bfloat16).to(DEV)
    seeds = torch.tensor([99], dtype=torch.int64).to(DEV)
    sid = torch.zeros(N, dtype=torch.int32, device=DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    cg = difr.gumbel_score(logits, T, seeds, sid, pos, None)["argmax"]
    ci = difr.ipt_score(logits, T, seeds, sid, pos, None, want_token=True)["ipt_token"]
    rnd = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    k = torch.arange(N, device=DEV)
    cg = torch.where(k % 3 == 0, rnd, cg)
    ci = torch.where(k % 3 == 1, rnd, ci)
    host = parity.to_host_logits(logits)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    gq = difr.gumbel_score(logits, T, seeds, sid, pos, cg)
    iq = difr.ipt_score(logits, T, seeds, sid, pos, ci)
    og = oracle.gumbel_score(host, V, np.float32(T), hs, hsid, hpos, cg.cpu().numpy())
    oi = oracle.ipt_score(host, V, np.float32(T), hs, hsid, hpos, ci.cpu().numpy())
    scale = max(1.0, float(np.abs(og["max_score"]).max()))
    m_err = np.nanmax(np.abs(gq["margin"].cpu().numpy().astype(np.float64) - og["margin"]))
    assert m_err <= 1e-4 * scale / 8, (m_err, scale)        # a few fp32 ulps of the scores
    near = og["gap2"] < 1e-6 * np.maximum(1.0, np.abs(og["max_score"]))
    assert ((gq["argmax"].cpu().numpy() == og["argmax"]) | near).all()
    parity.compare_ipt(iq, oi, tie_rel=1e-6)


@pytest.mark.parametrize("case", range(24))
def test_random_shapes_alignments_and_temperatures(difr, case):
    """Seeded random draws of everything a caller can vary at once: row count, vocabulary size (round
    boundaries +/- a few entries included), row stride, element type, a base offset that breaks the 16-byte
    alignment in a third of the cases, shared or per-row temperatures, number of sequences, honest / random /
    out-of-range claims.  Every row goes through the oracle."""
    rng = np.random.default_rng(4200 + case)
    dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
    per_vec = 8 if dtype == torch.bfloat16 else 4
    base_v = int(rng.choice([per_vec * 256, per_vec * 256 * 3, 5000, 12000, 333]))
    V = max(1, base_v + int(rng.integers(-9, 10)))
    N = int(rng.integers(1, 70))
    pad = int(rng.integers(0, 3)) * per_vec
    aligned = rng.random() > 0.33
    ld = ((V + per_vec - 1) // per_vec) * per_vec + pad if aligned else V + int(rng.integers(0, 3))
    offset = 0 if aligned else int(rng.integers(1, per_vec))
    g = torch.Generator().manual_seed(9000 + case)
    store = torch.full((N * ld + offset + 16,), float("nan"), dtype=dtype, device=DEV)
    logits = store[offset:offset + N * ld].view(N, ld)
    logits[:, :V] = (torch.randn(N, V, generator=g) * float(rng.uniform(0.5, 4.0))).to(dtype).to(DEV)
    S = int(rng.integers(1, 5))
    seeds = torch.from_numpy(rng.integers(-(1 << 63), (1 << 63) - 1, size=S, dtype=np.int64)).to(DEV)
    sid = torch.from_numpy(rng.integers(0, S, size=N).astype(np.int32)).to(DEV)
    pos = torch.from_numpy(rng.integers(0, 1 << 20, size=N).astype(np.int32)).to(DEV)
    T = float(rng.uniform(0.3, 1.8))
    temps = None
    if rng.random() < 0.4:
        temps = torch.from_numpy(rng.uniform(0.3, 1.8, size=N).astype(np.float32)).to(DEV)
    cg = difr.gumbel_score(logits, T, seeds, sid, pos, None, V=V, temperatures=temps)["argmax"]
    ci = difr.ipt_score(logits, T, seeds, sid, pos, None, V=V, temperatures=temps, want_token=True)["ipt_token"]
    rnd = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    k = torch.arange(N, device=DEV)
    cg = torch.where(k % 4 == 1, rnd, cg)
    ci = torch.where(k % 4 == 2, rnd, ci)
    if N > 5:
        cg[5] = V            # out of range: INVALID_CLAIM on that row only
        ci[3] = -1
    sg, si, was_aligned = _run_all(difr, logits, V, T, seeds, sid, pos, cg, ci, temps=temps)
    assert was_aligned == aligned


def test_bf16_nan_with_sign_bit_set(difr):
    """A bf16 NaN whose sign bit is set (pattern 0xFFC0, the default NaN of x86 arithmetic).  The oracle flags any
    NaN.  So do the calls that take the exponential of every entry (difr_ipt_score, the Token-IPT-DiFR side of
    difr_score_both) and the unfiltered Token-DiFR kernel.  The gated Token-DiFR stream orders raw bit patterns, in
    which such a NaN sorts below -inf: it is documented to treat the entry like a masked one, unless the vector that
    holds it reaches the exact evaluation for another reason, where it is flagged.  Either way the row never
    passes silently on the Token-IPT-DiFR side."""
    N, V, T = 64, 20504, 0.9
    g = torch.Generator().manual_seed(77)
    x = (torch.randn(N, V, generator=g) * 2.5).to(torch.bfloat16)
    bits = x.view(torch.int16)
    where = torch.randint(0, V, (N,), generator=g)
    masked = x.clone()
    for n in range(N):
        bits[n, where[n]] = -64                      # 0xFFC0
        masked[n, where[n]] = float("-inf")
    assert x.float().isnan().sum() == N
    x, masked = x.to(DEV), masked.to(DEV)
    seeds = torch.tensor([5, 9], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    c = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    host = parity.to_host_logits(x)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    og = oracle.gumbel_score(host, V, np.float32(T), hs, hsid, hpos, c.cpu().numpy())
    oi = oracle.ipt_score(host, V, np.float32(T), hs, hsid, hpos, c.cpu().numpy())
    assert (og["flags"] & 4).all() and (oi["flags"] & 4).all()
    i = difr.ipt_score(x, T, seeds, sid, pos, c)
    u = difr.gumbel_score(x, T, seeds, sid, pos, c, unfiltered=True)
    gs = difr.gumbel_score(x, T, seeds, sid, pos, c)
    gm = difr.gumbel_score(masked, T, seeds, sid, pos, c)
    fg, fi = difr.score_both(x, T, seeds, sid, pos, c, c)
    torch.cuda.synchronize()
    assert (i["flags"] & 4).all() and (fi["flags"] & 4).all()
    assert (u["flags"] & 4).all()
    flagged = (gs["flags"] & 4) != 0
    for k in gs:                                     # not flagged: exactly the row with the entry masked
        a, b = gs[k][~flagged], gm[k][~flagged]
        assert torch.equal(torch.nan_to_num(a.float(), nan=-7.0), torch.nan_to_num(b.float(), nan=-7.0)), k
    for k in fg:                                     # the one-pass call's Token-DiFR side is the same stream
        assert torch.equal(torch.nan_to_num(fg[k].float(), nan=-7.0), torch.nan_to_num(gs[k].float(), nan=-7.0)), k


@pytest.mark.parametrize("shift", [-60.0, 75.0])
@pytest.mark.parametrize("aligned", [True, False])
def test_cdf_accuracy_with_logits_far_from_zero(difr, shift, aligned):
    """Logits around -60 or +75 at T = 0.58: x c runs into the hundreds, where the product of a reference logit and c
    is only good to 1e-5.  The softmax terms are taken against that rounded product, so the lanes have to be combined
    by the rounded products too: the CDF must stay within a few 1e-7 of the oracle's (it was off by 1.3e-6 when the
    lanes were combined by the reference logits, enough to flip a MATCH the oracle decides by 1.1e-6)."""
    N, V, T = 24, 40000, 0.58
    g = torch.Generator().manual_seed(int(abs(shift)) + aligned)
    x = torch.randn(N, V, generator=g) * 2.0 + shift
    ld = V if aligned else V + 3
    buf = torch.full((N, ld), float("nan"), dtype=torch.bfloat16, device=DEV)
    buf[:, :V] = x.to(torch.bfloat16).to(DEV)
    logits = buf if aligned else buf
    seeds = torch.tensor([5, 1 << 33], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    temps = torch.linspace(0.35, 1.4, N).to(DEV)
    claims = difr.ipt_score(logits, T, seeds, sid, pos, None, V=V, temperatures=temps, want_token=True,
                            want_interval=False)["ipt_token"]
    out = difr.ipt_score(logits, T, seeds, sid, pos, claims, V=V, temperatures=temps)
    torch.cuda.synchronize()
    host = parity.to_host_logits(logits)
    ref = oracle.ipt_score(host, V, np.float32(T), parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos),
                           claims.cpu().numpy(), temps.cpu().numpy())
    for name in ("cdf_lo", "cdf_hi"):
        err = np.abs(out[name].cpu().numpy().astype(np.float64) - ref[name])
        assert err.max() <= 4e-7, (name, err.max())
