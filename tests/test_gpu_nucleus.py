"""GPU parity of the nucleus over the whole vocabulary (difr_ipt_score_filtered with top_k = 0, and the filter
threshold difr_gumbel_likelihood uses with top_k = 0) against the oracle.

Whether the marginal token of a nucleus of thousands of tokens is still inside is decided by a cumulative mass
that the GPU forms from fp32 exponentials and the oracle in double.  What can be PROVEN of the GPU's sum is the
per-term bound (the exponent of a term is rounded to fp32: up to 7e-7 relative for the small terms), so the
kept-set size must lie between the oracle's sizes at top_p -/+ 2e-6 and equal the oracle's wherever those two
agree.  The per-term errors differ from one logit value to the next and largely cancel, so the size nearly
always IS the oracle's: the rows where it is not are counted (`differs`), and so are the rows that the much
narrower width 1e-7 would leave in doubt.  Interval ends and the distance must agree within 1e-4 absolute (the
contract of the unfiltered estimator), which the mass of the few tokens in doubt (< 1e-5) does not touch."""
import sys

import numpy as np
import pytest
import torch

import oracle
import parity
from paper_2511_02620_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS_P = 2e-6          # proven width
EPS_P_NARROW = 1e-7   # reported only


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def difr():
    import paper_2511_02620_amd as m
    m.load_library()
    return m


def _oracle(host, V, T, seeds, sid, pos, claims, p, temps):
    return oracle.ipt_filtered_score(host, V, np.float32(T), parity.seeds_u64(seeds), sid.cpu().numpy(),
                                     parity.positions_u32(pos), None if claims is None else claims.cpu().numpy(), 0,
                                     float(p), temperatures=None if temps is None else temps.cpu().numpy(), sigma=0.02)


def _compare(difr, logits, V, T, seeds, sid, pos, claims, p, temps=None):
    eps_p = EPS_P
    out = difr.ipt_score_filtered(logits, T, seeds, sid, pos, claims, top_k=0, top_p=p, temperatures=temps, V=V,
                                  want_token=True, want_log_mass=True, sigma=0.02)
    torch.cuda.synchronize()
    plain = difr.ipt_score_filtered(logits, T, seeds, sid, pos, claims, top_k=0, top_p=p, temperatures=temps, V=V,
                                    want_log_mass=True, sigma=0.02)
    for name in ("dist", "cdf_lo", "cdf_hi", "u", "log_mass", "kept"):  # asking for the token changes nothing else
        assert torch.equal(out[name].view(torch.int32), plain[name].view(torch.int32)), name
    assert torch.equal(out["flags"] & ~8, plain["flags"])              # (but for the second-pass flag)
    tok = out.pop("ipt_token").cpu().numpy()
    host = parity.to_host_logits(logits)
    p32 = float(np.float32(p))
    ref = _oracle(host, V, T, seeds, sid, pos, claims, p32, temps)
    lo = _oracle(host, V, T, seeds, sid, pos, claims, p32 - eps_p, temps)["kept"]
    hi = _oracle(host, V, T, seeds, sid, pos, claims, p32 + eps_p, temps)["kept"]
    kept = out["kept"].cpu().numpy()
    assert (kept >= 0).all(), "undetermined rows"
    assert (kept >= lo).all() and (kept <= hi).all(), np.nonzero((kept < lo) | (kept > hi))[0][:10]
    sure = lo == hi
    assert (kept[sure] == ref["kept"][sure]).all()
    # rows whose kept set is the oracle's: the full comparison (log-mass included).  Rows in doubt differ from the
    # oracle by the marginal token(s): interval ends and distance within the 1e-4 contract, nothing finer.
    st = {}
    if sure.any():
        idx = torch.from_numpy(np.nonzero(sure)[0]).to(DEV)
        st = parity.compare_ipt({k2: v[idx] for k2, v in out.items() if k2 != "kept"},
                                {k2: v[sure] for k2, v in ref.items()}, log_mass_sigma=0.02)
    # (a marginal token is the least probable member of a set of `kept` tokens, so it holds at most 1 / kept of the
    # renormalised mass: that much an interval end may move per token in doubt - far below 1e-4 unless K is small and
    # made of ties, e.g. a constant row cut at exactly a whole number of tokens)
    slack = 1e-4 + (hi - lo)[~sure].astype(np.float64) / np.maximum(lo[~sure], 1)
    for name in ("cdf_lo", "cdf_hi", "dist"):
        g_, r_ = out[name].cpu().numpy().astype(np.float64)[~sure], ref[name][~sure]
        both_nan = np.isnan(g_) & np.isnan(r_)
        assert (both_nan | (np.abs(g_ - r_) <= slack)).all(), name
    # the sampler's own token, on the rows whose kept set is the oracle's: equal, except where u sits on a CDF step
    # (then the oracle's interval of the GPU's token touches u); a row the library gave up on has none
    flags = out["flags"].cpu().numpy()
    excused = 0
    for r in np.nonzero(sure)[0]:
        if flags[r] & 4:
            assert tok[r] == -1
        elif tok[r] != ref["ipt_token"][r]:
            one = oracle.ipt_filtered_score(host[r:r + 1], V, np.float32(T) if temps is None else float(temps[r]),
                                            parity.seeds_u64(seeds), sid.cpu().numpy()[r:r + 1],
                                            parity.positions_u32(pos)[r:r + 1], np.array([tok[r]], np.int32), 0, p32)
            assert one["dist"][0] < 1e-5 and one["cdf_hi"][0] > one["cdf_lo"][0], (r, tok[r], ref["ipt_token"][r])
            excused += 1
    st["token_excused"] = excused
    st["mean_kept"] = float(kept.mean())
    st["rows_in_doubt"] = int((~sure).sum())
    st["differs"] = int((kept != ref["kept"]).sum())
    lo_n = _oracle(host, V, T, seeds, sid, pos, claims, p32 - EPS_P_NARROW, temps)["kept"]
    hi_n = _oracle(host, V, T, seeds, sid, pos, claims, p32 + EPS_P_NARROW, temps)["kept"]
    st["in_doubt_at_1e-7"] = int((lo_n != hi_n).sum())
    # a row whose cut the oracle itself moves within 1e-7 of top_p - the accuracy of one fp32 exponential - may go
    # either way (a constant row cut at a whole number of tokens does); of the others, nearly all must be the oracle's
    st["differs_beyond_1e-7"] = int(((kept != ref["kept"]) & (lo_n == hi_n)).sum())
    assert st["differs_beyond_1e-7"] <= max(1, kept.shape[0] // 20)
    out["ipt_token"] = torch.from_numpy(tok).to(DEV)
    return st, out


@pytest.mark.parametrize("dtype,V,p,kind", [
    (torch.bfloat16, 20504, 0.95, "normal"),       # thousands of tokens in the nucleus, many equal bf16 logits
    (torch.bfloat16, 20504, 0.5, "normal"),
    (torch.bfloat16, 20504, 0.9, "peaked"),        # a handful of tokens
    (torch.bfloat16, 2051, 0.99, "normal"),        # ragged last vector
    (torch.bfloat16, 300, 0.7, "normal"),          # a single, partly filled round
    (torch.float32, 5003, 0.9, "normal"),          # fp32 keys: more search passes
    (torch.float32, 5003, 0.95, "coarse"),         # fp32 storage, few distinct values: long runs of ties at the cut
    (torch.bfloat16, 16384, 0.8, "masked"),        # half of the vocabulary at -inf
    (torch.bfloat16, 40000, 0.9, "coarse"),        # thousands of tokens share the logit at the cut: no sorting, a division
    (torch.float32, 40000, 0.6, "coarse"),
])
def test_nucleus_every_row(difr, dtype, V, p, kind):
    N = 48
    g = torch.Generator().manual_seed(31 + V + int(p * 100))
    ld = ((V + 7) // 8) * 8
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)
    x = torch.randn(N, V, generator=g) * (6.0 if kind == "peaked" else 2.0)
    if kind == "coarse":
        x = torch.round(x * 2) / 2
    if kind == "masked":
        x[:, ::2] = float("-inf")
    logits[:, :V] = x.to(dtype).to(DEV)
    seeds = torch.tensor([11, 1 << 50], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    T = 0.9
    # claims: the top token, a random token (mostly outside a small nucleus), an out-of-range one
    claims = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    top = logits[:, :V].float().argmax(dim=1).to(torch.int32)
    claims = torch.where(torch.arange(N, device=DEV) % 3 == 0, top, claims)
    claims[5] = V
    st, out = _compare(difr, logits, V, T, seeds, sid, pos, claims, p)
    say("nucleus", dtype, V, p, kind, st)
    assert not (out["flags"] & 4).any()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("layout", ["ascending", "descending", "head_masked", "constant", "two_values",
                                    "tiny_head_span", "far_below_head", "huge_tail"])
def test_nucleus_first_round_unlike_the_row(difr, dtype, layout):
    """The search lays its first bins over the values met in the first 2048 (bf16) or 1024 (fp32) entries and takes
    its exponent reference from them; rows whose beginning says nothing about the rest - or something misleading -
    must come out the same: sorted either way, a masked beginning, one or two distinct values, a beginning whose
    values span next to nothing, a maximum so far above the beginning that the pass has to start again, and a
    beginning of outliers far above a flat rest."""
    N, V = 24, 9000
    g = torch.Generator().manual_seed(77 + len(layout) + (dtype == torch.float32))
    x = torch.randn(N, V, generator=g) * 2.0
    T = 0.9
    if layout == "ascending":
        x = x.sort(dim=1).values
    elif layout == "descending":
        x = x.sort(dim=1, descending=True).values
    elif layout == "head_masked":
        x[:, :2300] = float("-inf")
    elif layout == "constant":
        x[:] = -1.25
    elif layout == "two_values":
        x = torch.where(torch.rand(N, V, generator=g) < 0.01, torch.tensor(3.0), torch.tensor(-2.0))
    elif layout == "tiny_head_span":
        x[:, :2300] = 1.0
        x[:, 7] = 1.0 + 2.0 ** -7       # the next bf16 (and an fp32) value above 1
    elif layout == "far_below_head":
        x[:, :2300] -= 120.0             # (M - R) c is far beyond what an fp32 term can hold
    elif layout == "huge_tail":
        x = x * 0.05 - 30.0
        x[:, :64] = torch.randn(N, 64, generator=g) + 5.0
    ld = ((V + 7) // 8) * 8
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)
    logits[:, :V] = x.to(dtype).to(DEV)
    seeds = torch.tensor([3, 1 << 40], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    claims = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    top = logits[:, :V].float().argmax(dim=1).to(torch.int32)
    claims = torch.where(torch.arange(N, device=DEV) % 2 == 0, top, claims)
    for p in (0.3, 0.9, 0.99):
        st, out = _compare(difr, logits, V, T, seeds, sid, pos, claims, p)
        say("nucleus layout", layout, dtype, p, st)
        assert not (out["flags"] & 4).any()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_nucleus_cut_on_a_tie_of_large_logits(difr, dtype):
    """Logits in the hundreds at T = 0.6: the exponent (x - R) log2(e) / T has to come from the difference, not from two
    products of that size.  The two largest logits are equal and hold half of the mass each, so top_p = 0.5 needs both
    (the rest of the row adds a few 1e-6 to the total): a mass that is off by 1e-5 keeps one."""
    N, V = 32, 1017
    g = torch.Generator().manual_seed(91)
    x = (torch.randn(N, V, generator=g) * 60.0).round()
    top = x.max(dim=1).values + 7.0
    for r in range(N):
        i, j = torch.randperm(V, generator=g)[:2].tolist()
        x[r, i] = x[r, j] = top[r]
    E = 8 if dtype == torch.bfloat16 else 4
    ld = ((V + E - 1) // E) * E
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)
    logits[:, :V] = x.to(dtype).to(DEV)
    seeds = torch.tensor([17], dtype=torch.int64).to(DEV)
    sid = torch.zeros(N, dtype=torch.int32, device=DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    claims = logits[:, :V].float().argmax(dim=1).to(torch.int32)
    for p in (0.5, 0.4, 0.999):
        st, out = _compare(difr, logits, V, 0.6, seeds, sid, pos, claims, p)
        say("nucleus tie of large logits", dtype, p, st)
        if p == 0.5:
            assert (out["kept"] == 2).all()


def test_nucleus_zipf_rows_and_per_row_temperatures(difr):
    """C2-class rows (V = 128256, Zipf profile): flat distributions whose 0.95-nucleus holds tens of thousands of
    tokens; per-row temperatures."""
    wl = W.scaled(W.C2_3B, S=2, L=24, chunk_rows=48)
    ver, prov = wl.logits_chunk(0, DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    temps = torch.linspace(0.4, 1.2, wl.N, device=DEV)
    claims = difr.ipt_score(prov, 1.0, seeds, sid, pos, None, temperatures=temps, want_token=True, want_interval=False)["ipt_token"]
    for p in (0.9, 0.95):
        st, out = _compare(difr, ver, wl.V, 1.0, seeds, sid, pos, claims, p, temps=temps)
        say("nucleus C2 rows p", p, st)


@pytest.mark.parametrize("dtype,kind", [(torch.bfloat16, "normal"), (torch.float32, "coarse"), (torch.bfloat16, "coarse")])
def test_nucleus_sampling_mode_round_trip(difr, dtype, kind):
    """No claims: the call returns the sampler's token under the bare nucleus.  Scored as claims, those tokens match
    on every row, with distance 0, and come back as the sampler's token."""
    N, V = 64, 12296
    g = torch.Generator().manual_seed(5 + len(kind))
    x = torch.randn(N, V, generator=g) * 2.0
    if kind == "coarse":
        x = torch.round(x * 2) / 2
    logits = x.to(dtype).to(DEV)
    seeds = torch.tensor([3, 1 << 40, 99], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 3).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    for p in (0.5, 0.97):
        drawn = difr.ipt_score_filtered(logits, 0.8, seeds, sid, pos, None, top_k=0, top_p=p, want_token=True)
        tok = drawn["ipt_token"]
        assert ((tok >= 0) & (tok < V)).all()
        assert (drawn["flags"] & 2).all()  # no claim: INVALID_CLAIM, the scores are NaN
        back = difr.ipt_score_filtered(logits, 0.8, seeds, sid, pos, tok, top_k=0, top_p=p, want_token=True)
        torch.cuda.synchronize()
        assert (back["flags"] & 1).all() and (back["dist"] == 0).all()
        assert torch.equal(back["ipt_token"], tok)
        assert torch.equal(back["kept"], drawn["kept"])
        # the token lies inside the nucleus: its logit is no smaller than the smallest kept one
        st, _ = _compare(difr, logits, V, 0.8, seeds, sid, pos, tok, p)
        say("nucleus sampling", dtype, kind, p, st)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("p", [0.6, 0.3, 0.2, 0.99])
def test_nucleus_signed_zeros_tie_by_index(difr, dtype, p):
    """-0 and +0 are the same logit: where the cut falls among zeros of both signs, the ties enter the nucleus in
    index order whatever their sign (p = 0.6 and 0.3; at 0.2 the cut lies above the zeros, at 0.99 below them)."""
    N, V = 32, 4000
    g = torch.Generator().manual_seed(17)
    x = torch.full((N, V), -3.0)
    for r in range(N):
        perm = torch.randperm(V, generator=g)
        x[r, perm[:100]] = 2.0
        z = perm[100:2100]
        x[r, z] = torch.where(torch.rand(2000, generator=g) < 0.5, torch.tensor(0.0), torch.tensor(-0.0))
    logits = x.to(dtype).to(DEV)
    assert (torch.signbit(logits) & (logits == 0)).any() and (~torch.signbit(logits) & (logits == 0)).any()
    seeds = torch.tensor([21], dtype=torch.int64).to(DEV)
    sid = torch.zeros(N, dtype=torch.int32, device=DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    claims = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    st, out = _compare(difr, logits, V, 1.0, seeds, sid, pos, claims, p)
    say("nucleus signed zeros", dtype, p, st)
    assert st["rows_in_doubt"] == 0 and st["rows"] == N
    # and in sampling mode
    tok = difr.ipt_score_filtered(logits, 1.0, seeds, sid, pos, None, top_k=0, top_p=p, want_token=True)["ipt_token"]
    st, _ = _compare(difr, logits, V, 1.0, seeds, sid, pos, tok, p)
    assert st["match_excused"] == 0 and st["token_excused"] == 0


def test_likelihood_with_a_whole_vocabulary_nucleus(difr):
    """top_k = 0, top_p < 1 in difr_gumbel_likelihood: tau is the smallest logit of the nucleus; it must be the
    oracle's at top_p, or lie between the oracle's at top_p -/+ 2e-6; pi must then agree wherever tau does."""
    N, V = 40, 20504
    g = torch.Generator().manual_seed(77)
    logits = (torch.randn(N, V, generator=g) * 2.0).to(torch.bfloat16).to(DEV)
    seeds = torch.tensor([5], dtype=torch.int64).to(DEV)
    sid = torch.zeros(N, dtype=torch.int32, device=DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    cg = difr.gumbel_score(logits, 0.8, seeds, sid, pos, None, want_scores=False)["argmax"]
    z = torch.randn(128, generator=g, dtype=torch.float32)
    out = difr.gumbel_likelihood(logits, 0.8, seeds, sid, pos, cg, z.to(DEV), top_k=0, top_p=0.9, s=8, sigma=0.4)
    torch.cuda.synchronize()
    host = parity.to_host_logits(logits)
    args = (host, V, np.float32(0.8), parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos), cg.cpu().numpy())
    p32 = float(np.float32(0.9))
    ref = oracle.likelihood(*args, 0, p32, 8, 0.4, z.numpy().astype(np.float64))
    lo = oracle.likelihood(*args, 0, p32 + EPS_P, 8, 0.4, z.numpy().astype(np.float64))["tau"]   # more mass: lower threshold
    hi = oracle.likelihood(*args, 0, p32 - EPS_P, 8, 0.4, z.numpy().astype(np.float64))["tau"]
    tau = out["tau"].cpu().numpy().astype(np.float64)
    assert (tau >= lo).all() and (tau <= hi).all()
    same = tau == ref["tau"]
    assert same[lo == hi].all() and same.mean() > 0.95
    pi = out["pi"].cpu().numpy().astype(np.float64)
    assert np.abs(pi[same] - ref["pi"][same]).max() < 1e-4
    say("likelihood with nucleus: tau equal on %d of %d rows, pi err %.2e" % (same.sum(), N, np.abs(pi[same] - ref["pi"][same]).max()))


@pytest.mark.parametrize("case", range(16))
def test_nucleus_random_shapes(difr, case):
    """Seeded random vocabulary sizes (round boundaries +/- a few entries), element types, spreads of the logits,
    temperatures (shared or per row) and top_p values; every row against the oracle."""
    rng = np.random.default_rng(7700 + case)
    dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
    per_vec = 8 if dtype == torch.bfloat16 else 4
    V = max(2, int(rng.choice([per_vec * 256, per_vec * 256 * 2, 3000, 9000, 150])) + int(rng.integers(-5, 6)))
    ld = ((V + per_vec - 1) // per_vec) * per_vec + int(rng.integers(0, 2)) * per_vec
    N = int(rng.integers(1, 40))
    g = torch.Generator().manual_seed(100 + case)
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)
    logits[:, :V] = (torch.randn(N, V, generator=g) * float(rng.uniform(0.3, 5.0)) + float(rng.uniform(-20, 20))).to(dtype).to(DEV)
    S = int(rng.integers(1, 4))
    seeds = torch.from_numpy(rng.integers(-(1 << 63), (1 << 63) - 1, size=S, dtype=np.int64)).to(DEV)
    sid = torch.from_numpy(rng.integers(0, S, size=N).astype(np.int32)).to(DEV)
    pos = torch.from_numpy(rng.integers(0, 1 << 20, size=N).astype(np.int32)).to(DEV)
    T = float(rng.uniform(0.2, 1.6))
    temps = torch.from_numpy(rng.uniform(0.2, 1.6, size=N).astype(np.float32)).to(DEV) if rng.random() < 0.4 else None
    p = float(rng.choice([0.1, 0.5, 0.8, 0.9, 0.95, 0.99, 0.999]))
    claims = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    top = logits[:, :V].float().argmax(dim=1).to(torch.int32)
    claims = torch.where(torch.arange(N, device=DEV) % 2 == 0, top, claims)
    st, out = _compare(difr, logits, V, T, seeds, sid, pos, claims, p, temps=temps)
    say("nucleus random", case, dtype, V, "p", p, st)
