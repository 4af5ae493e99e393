"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (one launch over the
whole resident batch), with the oracle on EVERY row of the stored-logit configurations.

The batch is built chunk by chunk.  For each chunk of 512 rows the oracle's two samplers run on the prover
logits (these are the honest claims: no oracle input is produced by the HIP path), the library's samplers
run on the same chunk and are compared with them row by row, the configuration's dishonest-token recipe is
applied, and the oracle scores the claims against the verifier logits.  After the last chunk the library
scores the whole resident batch in one launch and every row is compared with the oracle; pooling, thresholds
(calibrated from the ORACLE's per-sequence means) and flags are compared for every sequence.  Estimators
whose oracle sorts the whole vocabulary per row (likelihood, filtered IPT, nucleus, admissible set) are
compared on a seeded sample of rows and by properties on all rows."""
import gc
import time

import numpy as np
import pytest
import torch

import oracle
import parity
from paper_2511_02620_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SIGMA_IPT = 0.01


def f32(x):
    return float(np.float32(x))


@pytest.fixture(scope="module")
def difr():
    assert torch.cuda.is_available()
    import paper_2511_02620_amd as d

    d.load_library()
    return d


@pytest.fixture
def say(capsys):
    """Progress lines that are not held back by pytest's capture (a whole-batch oracle pass takes minutes)."""
    def _say(*a):
        with capsys.disabled():
            print(*a, flush=True)
    return _say


def _host_bits(pinned, t):
    pinned.copy_(t)
    torch.cuda.synchronize()
    return pinned.view(torch.int16).numpy().view(np.uint16)


def _merge(total, st):
    for k, v in st.items():
        if k.endswith("_err"):
            total[k] = max(total.get(k, 0.0), v)
        else:
            total[k] = total.get(k, 0) + v
    return total


def _build_with_oracle(difr, wl, deep_rows, say):
    """Resident verifier logits, claims for both estimators, the oracle's outputs for every row, and host copies
    of the verifier logits of `deep_rows`."""
    N, V, R = wl.N, wl.V, wl.chunk_rows
    T = wl.temperature
    logits = torch.empty(N, V, dtype=wl.dtype, device=DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    cg, ci = np.empty(N, np.int32), np.empty(N, np.int32)
    og = dict(margin=np.empty(N), argmax=np.empty(N, np.int32), max_score=np.empty(N), claimed_score=np.empty(N),
              gap2=np.empty(N), flags=np.empty(N, np.uint8))
    oi = dict(u=np.empty(N), cdf_lo=np.empty(N), cdf_hi=np.empty(N), dist=np.empty(N), ipt_token=np.empty(N, np.int32),
              log_mass=np.empty(N), edge=np.empty(N), flags=np.empty(N, np.uint8))
    deep = np.asarray(deep_rows, dtype=np.int64)
    deep_host = np.empty((len(deep), V), dtype=np.uint16)
    pin_v = torch.empty(R, V, dtype=wl.dtype, pin_memory=True)
    pin_p = torch.empty(R, V, dtype=torch.bfloat16, pin_memory=True)
    assert wl.prover_bf16
    sampler_g, sampler_i = {}, {}
    t0 = time.time()
    for c in range(wl.n_chunks):
        r0, r1 = c * R, (c + 1) * R
        ver, prov = wl.logits_chunk(c, DEV)
        logits[r0:r1] = ver
        # the library's samplers on the prover logits (sampling mode: no claims)
        hip_g = difr.gumbel_score(prov, T, seeds, sid[r0:r1], pos[r0:r1], None)
        hip_i = difr.ipt_score(prov, T, seeds, sid[r0:r1], pos[r0:r1], None, want_token=True)
        ph = _host_bits(pin_p, prov)
        # the oracle's samplers on the same bytes: the honest claims
        sg = oracle.gumbel_score(ph, V, f32(T), hs, hsid[r0:r1], hpos[r0:r1])
        si = oracle.ipt_score(ph, V, f32(T), hs, hsid[r0:r1], hpos[r0:r1])
        _merge(sampler_g, parity.compare_gumbel(hip_g, sg))
        _merge(sampler_i, parity.compare_ipt(hip_i, si, ph, V, (f32(T), hs, hsid[r0:r1], hpos[r0:r1])))
        # the configuration's dishonest-token recipe (input generation, no method arithmetic)
        cgc = wl.mutate_claims(c, torch.from_numpy(sg["argmax"].copy()).to(DEV), ver).cpu().numpy()
        cic = wl.mutate_claims(c, torch.from_numpy(si["ipt_token"].copy()).to(DEV), ver).cpu().numpy()
        cg[r0:r1], ci[r0:r1] = cgc, cic
        # the oracle's scores of those claims against the verifier logits
        vh = _host_bits(pin_v, ver)
        o1 = oracle.gumbel_score(vh, V, f32(T), hs, hsid[r0:r1], hpos[r0:r1], cgc)
        o2 = oracle.ipt_score(vh, V, f32(T), hs, hsid[r0:r1], hpos[r0:r1], cic, sigma=SIGMA_IPT)
        for k in og:
            og[k][r0:r1] = o1[k]
        for k in oi:
            oi[k][r0:r1] = o2[k]
        inside = np.nonzero((deep >= r0) & (deep < r1))[0]
        if inside.size:
            deep_host[inside] = vh[deep[inside] - r0]
        del ver, prov
        if (c + 1) % 16 == 0 or c + 1 == wl.n_chunks:
            say("  %s T=%g: oracle through row %d of %d (%.0f s, %d oracle threads)" % (wl.name, T, r1, N, time.time() - t0,
                                                                                        oracle.num_threads()))
    say("  %s T=%g samplers, library against oracle on all %d rows: gumbel %s ipt %s" % (wl.name, T, N, sampler_g, sampler_i))
    assert sampler_g["argmax_excused"] <= 1e-3 * N and sampler_i["token_excused"] <= 2e-2 * N
    return (logits, seeds, sid, pos, torch.from_numpy(cg).to(DEV), torch.from_numpy(ci).to(DEV)), og, oi, deep_host, (hs, hsid, hpos)


def _same(a, b, what, mask_slow=False):
    for k in a:
        x, y = a[k], b[k]
        if mask_slow and k == "flags":
            x, y = x & 0xF7, y & 0xF7
        if x.dtype.is_floating_point:
            x, y = torch.nan_to_num(x, nan=-7.0), torch.nan_to_num(y, nan=-7.0)
        assert torch.equal(x, y), (what, k, int((x != y).sum()))


def _check_all_rows(g, i):
    """Properties that hold for every row whatever the inputs."""
    m, fl = g["margin"], g["flags"]
    assert bool((m >= 0).all()) and bool(((fl & 6) == 0).all())
    assert bool(((fl & 1) == 1).eq(m == 0).all())                 # MATCH <=> margin exactly 0 (ties aside)
    assert bool((g["max_score"] - g["claimed_score"] == m).all())
    d, a, b, u = i["dist"], i["cdf_lo"], i["cdf_hi"], i["u"]
    assert bool((d >= 0).all()) and bool((d < 1).all()) and bool((a <= b).all()) and bool((a >= 0).all())
    assert bool((b <= 1.0 + 1e-6).all()) and bool((u > 0).all()) and bool((u < 1).all())
    matched = (i["flags"] & 1) == 1
    assert bool((d[matched] == 0).all())
    expect = torch.clamp(torch.maximum(a - u, u - b), min=0)
    assert float((d - expect).abs().max()) <= 1e-6


def _score_every_row(difr, wl, batch, og, oi, host_args, tau_g, tau_i, say):
    """The timed launch configuration against the oracle on every row and every sequence."""
    logits, seeds, sid, pos, cg, ci = batch
    hs, hsid, hpos = host_args
    T = wl.temperature
    off = wl.seq_offsets().to(DEV)
    g = difr.gumbel_score(logits, T, seeds, sid, pos, cg)
    i = difr.ipt_score(logits, T, seeds, sid, pos, ci, want_token=True, want_log_mass=True, sigma=SIGMA_IPT)
    sg = difr.seq_reduce(g["margin"], g["flags"], off, tau_g)
    si = difr.seq_reduce(i["dist"], i["flags"], off, tau_i)
    g2 = difr.gumbel_score(logits, T, seeds, sid, pos, cg)           # same launch again: bit-identical
    i2 = difr.ipt_score(logits, T, seeds, sid, pos, ci, want_token=True, want_log_mass=True, sigma=SIGMA_IPT)
    torch.cuda.synchronize()
    _same(g, g2, "gumbel twice")
    _same(i, i2, "ipt twice")
    del g2, i2
    # the one-pass call the benchmark times returns the same outputs, bit for bit, on every row
    gb, ib = difr.score_both(logits, T, seeds, sid, pos, cg, ci, want_token=True, want_log_mass=True, sigma=SIGMA_IPT)
    torch.cuda.synchronize()
    _same(gb, g, "score_both gumbel")
    _same(ib, i, "score_both ipt")
    del gb, ib
    _check_all_rows(g, i)
    # every row against the oracle.  Tokens that differ are re-asked row by row from the resident logits.
    st_g = parity.compare_gumbel(g, og)
    tok_gpu, tok_ref = i["ipt_token"].cpu().numpy(), oi["ipt_token"]
    differ = np.nonzero(tok_gpu != tok_ref)[0]
    st_i = parity.compare_ipt({k: v for k, v in i.items() if k != "ipt_token"}, oi, log_mass_sigma=SIGMA_IPT)
    for r in differ:
        x = oracle.decode_row(parity.to_host_logits(logits[int(r)]))
        alt = oracle.ipt_row(x, f32(T), int(hs[hsid[r]]), int(hsid[r]), int(hpos[r]), int(tok_gpu[r]))
        assert alt["dist"] < parity.TIE_REL and alt["cdf_hi"] > alt["cdf_lo"], ("ipt_token beyond a near tie", int(r))
    st_i["token_excused"] = int(differ.size)
    say("  %s T=%g every row: gumbel %s" % (wl.name, T, st_g))
    say("  %s T=%g every row: ipt %s" % (wl.name, T, st_i))
    assert st_i["log_mass_beyond_bar"] == 0
    # pooling and flags of every sequence against the oracle's pooling of the oracle's scores
    pooled_stats = {}
    for o, pooled, tau, key, st in ((og, sg, tau_g, "margin", st_g), (oi, si, tau_i, "dist", st_i)):
        ref = oracle.seq_reduce(o[key], o["flags"], off.cpu().numpy(), np.float32(tau))
        st_s = pooled_stats[key] = parity.compare_seq(pooled, ref, float(tau), st["match_excused"])
        say("  %s T=%g pooled %s over %d sequences: %s" % (wl.name, T, key, wl.S, st_s))
    return g, i, sg, si, pooled_stats


def _sampled_estimators(difr, wl, batch, g, deep_rows, deep_host, host_args, say):
    """Estimators whose oracle sorts the vocabulary: every row by properties and against their one-pass forms,
    the oracle on the sampled rows."""
    logits, seeds, sid, pos, cg, ci = batch
    hs, hsid_all, hpos_all = host_args
    T = wl.temperature
    sel = torch.tensor(deep_rows, dtype=torch.int64, device=DEV)
    hsid, hpos = hsid_all[deep_rows], hpos_all[deep_rows]
    host = deep_host
    # admissible-set size on every row; the oracle's count on the sampled rows (an fp32 threshold decision:
    # the GPU's count must lie between the oracle's counts at delta -/+ 2e-5)
    a1 = difr.admissible_count(logits, T, seeds, sid, pos, g["max_score"], 1.0)
    a2 = difr.admissible_count(logits, T, seeds, sid, pos, g["max_score"], 2.5)
    torch.cuda.synchronize()
    assert (a1["count"] >= 1).all() and (a1["count"] <= a2["count"]).all()
    oa = oracle.admissible_count(host, wl.V, f32(T), hs, hsid, hpos, 2.5, tol=2e-5)
    ca = a2["count"][sel].cpu().numpy()
    assert (ca >= oa["count_lo"]).all() and (ca <= oa["count_hi"]).all()
    sure = oa["count_lo"] == oa["count_hi"]
    assert (ca[sure] == oa["count"][sure]).all()
    say("  %s T=%g admissible set at delta 2.5: mean size %.2f over all rows, %d of %d oracle rows near the threshold"
        % (wl.name, T, float(a2["count"].float().mean()), int((~sure).sum()), len(deep_rows)))
    # the same count from the one-pass call, with both scores: every row determined and equal to the two-pass count
    g1, i1, a3 = difr.score_both_admissible(logits, T, seeds, sid, pos, 2.5, cg, ci)
    torch.cuda.synchronize()
    assert torch.equal(a3["count"], a2["count"]), int((a3["count"] != a2["count"]).sum())
    _same(g1, g, "score_both_admissible gumbel")
    del g1, i1, a1, a3
    # Token-DiFR likelihood estimate with the paper's generation policy (top-k 50, top-p 0.95) on every row;
    # the oracle on the first 384 sampled rows (it sorts the whole vocabulary twice per row)
    z = torch.randn(256, generator=torch.Generator().manual_seed(5), dtype=torch.float32)
    lk = difr.gumbel_likelihood(logits, T, seeds, sid, pos, cg, z.to(DEV), top_k=50, top_p=0.95, s=16, sigma=0.3,
                                want_active=True)
    torch.cuda.synchronize()
    pi_all = lk["pi"]
    assert ((pi_all >= 0) & (pi_all <= 1)).all() and (lk["flags"] == 0).all()
    n_l = min(384, len(deep_rows))
    ssel = sel[:n_l]
    ol = oracle.likelihood(host[:n_l], wl.V, f32(T), hs, hsid[:n_l], hpos[:n_l], cg[ssel].cpu().numpy(), 50,
                           float(f32(0.95)), 16, float(f32(0.3)), z.double().numpy())
    assert np.array_equal(lk["tau"][ssel].cpu().numpy(), ol["tau"].astype(np.float32))
    diff = (lk["active"][ssel].cpu().numpy() != ol["active"]).any(axis=1)
    excused = diff & (ol["gap_s"] < 1e-5)
    assert not (diff & ~excused).any()
    perr = np.where(excused, 0.0, np.abs(lk["pi"][ssel].cpu().numpy().astype(np.float64) - ol["pi"]))
    assert perr.max() <= 1e-4
    say("  %s T=%g likelihood: mean pi %.4f over all rows, worst error %.3g on %d oracle rows, %d excused"
        % (wl.name, T, float(pi_all.mean()), perr.max(), n_l, int(excused.sum())))
    # Token-IPT-DiFR under the same filter, every row; the oracle on the same rows
    fi = difr.ipt_score_filtered(logits, T, seeds, sid, pos, ci, top_k=50, top_p=0.95)
    torch.cuda.synchronize()
    assert ((fi["dist"] >= 0) & (fi["dist"] < 1)).all() and (fi["flags"] & 6 == 0).all() and (fi["kept"] >= 1).all()
    ofi = oracle.ipt_filtered_score(host[:n_l], wl.V, f32(T), hs, hsid[:n_l], hpos[:n_l], ci[ssel].cpu().numpy(), 50,
                                    float(f32(0.95)))
    assert np.array_equal(fi["kept"][ssel].cpu().numpy(), ofi["kept"])
    st_f = parity.compare_ipt({k: v[ssel] for k, v in fi.items() if k != "kept"}, ofi)
    say("  %s T=%g filtered ipt: %s mean kept %.1f" % (wl.name, T, st_f, float(fi["kept"].float().mean())))
    # the two filtered estimators from one read of the logits: identical to the two calls on every row
    lk2, fi2 = difr.score_both_filtered(logits, T, seeds, sid, pos, cg, ci, z.to(DEV), top_k=50, top_p=0.95, s=16,
                                        sigma=0.3, want_active=True)
    torch.cuda.synchronize()
    _same(lk, lk2, "score_both_filtered likelihood")
    _same(fi, fi2, "score_both_filtered ipt")
    del lk2, fi2, lk, fi
    # the bare nucleus (no top-k): every row, the oracle on the first 128 sampled rows at top_p and top_p -/+ 2e-6
    # (what can be proven of a mass summed from fp32 exponentials); how many sizes equal the oracle's is reported,
    # and how many rows the narrower width 1e-7 would leave in doubt
    nu = difr.ipt_score_filtered(logits, T, seeds, sid, pos, ci, top_k=0, top_p=0.9)
    torch.cuda.synchronize()
    assert (nu["kept"] >= 1).all() and (nu["flags"] & 6 == 0).all()
    n_n = min(128, len(deep_rows))
    nsel = sel[:n_n]
    onu = [oracle.ipt_filtered_score(host[:n_n], wl.V, f32(T), hs, hsid[:n_n], hpos[:n_n], ci[nsel].cpu().numpy(), 0,
                                     float(f32(0.9)) + dp) for dp in (0.0, -2e-6, 2e-6, -1e-7, 1e-7)]
    kn = nu["kept"][nsel].cpu().numpy()
    assert (kn >= onu[1]["kept"]).all() and (kn <= onu[2]["kept"]).all()
    pinned = onu[1]["kept"] == onu[2]["kept"]
    assert (kn[pinned] == onu[0]["kept"][pinned]).all()
    for name in ("cdf_lo", "cdf_hi", "dist"):
        assert np.abs(nu[name][nsel].cpu().numpy().astype(np.float64) - onu[0][name]).max() <= 1e-4, name
    same = int((kn == onu[0]["kept"]).sum())
    say("  %s T=%g nucleus 0.9: mean kept %.0f over all rows; %d of %d oracle rows with the oracle's size; %d rows not pinned "
        "by the proven width 2e-6, %d by 1e-7" % (wl.name, T, float(nu["kept"].float().mean()), same, n_n, int((~pinned).sum()),
                                                  int((onu[3]["kept"] != onu[4]["kept"]).sum())))
    assert same >= n_n - max(1, n_n // 20)


def _deep_rows(wl, seed, n=512):
    rng = np.random.default_rng(seed)
    return sorted(set(int(r) for r in rng.integers(0, wl.N, size=n)) | {0, wl.N - 1})


@pytest.mark.parametrize("T", [1.0, 0.6])
def test_c3_full_size_every_row(difr, say, T):
    wl = W.C3_30B.with_temperature(T)
    deep = _deep_rows(wl, 31 + int(T * 10))
    say("C3 T=%g: %d rows x V=%d, oracle on every row" % (T, wl.N, wl.V))
    batch, og, oi, deep_host, host_args = _build_with_oracle(difr, wl, deep, say)
    tau_g, tau_i = 0.02, 0.001
    g, i, sg, si, _ = _score_every_row(difr, wl, batch, og, oi, host_args, tau_g, tau_i, say)
    _sampled_estimators(difr, wl, batch, g, deep, deep_host, host_args, say)
    match = float((g["flags"] & 1).float().mean())
    say("  C3 T=%g gumbel match rate %.4f, ipt match rate %.4f" % (T, match, float((i["flags"] & 1).float().mean())))
    assert match > 0.98                                 # bf16-level drift flips well under 2% of the samples
    del batch, g, i
    gc.collect()
    torch.cuda.empty_cache()


def test_c5_stego_audit_full_size_every_row(difr, say):
    wl = W.C5_STEGO
    stego = wl.stego_sequences()
    assert len(stego) == 3
    honest = [s for s in range(wl.S) if s not in stego]
    deep = _deep_rows(wl, 55, n=256)
    say("C5: %d rows x V=%d, oracle on every row" % (wl.N, wl.V))
    batch, og, oi, deep_host, host_args = _build_with_oracle(difr, wl, deep, say)
    # thresholds at FPR 1e-2 from the ORACLE's per-sequence means of the 253 honest sequences
    off = wl.seq_offsets().numpy()
    taus = {}
    for key, o in (("margin", og), ("dist", oi)):
        means = oracle.seq_reduce(o[key], o["flags"], off, np.float32(0.0))["seq_mean"]
        taus[key] = oracle.calibrate_threshold(means[honest], 1e-2)
        assert int((means[honest] > taus[key]).sum()) == 2          # floor(0.01 * 253)
    g, i, sg, si, pooled_stats = _score_every_row(difr, wl, batch, og, oi, host_args, taus["margin"], taus["dist"], say)
    for name, pooled, o in (("margin", sg, og), ("dist", si, oi)):
        tau = taus[name]
        fl = pooled["seq_flag"].cpu().numpy()
        mean = pooled["seq_mean"].cpu().numpy()
        ref = oracle.seq_reduce(o[name], o["flags"], off, np.float32(tau))
        say("  C5", name, "tau %.6g (oracle-calibrated)" % tau, "stego means", mean[stego], "flagged", fl[stego].tolist(),
            "honest flagged", int(fl[honest].sum()), "oracle flags the same", bool(np.array_equal(fl, ref["seq_flag"])))
        assert np.array_equal(fl, (~(mean <= np.float32(tau))).astype(np.uint8))
        assert ref["seq_flag"][stego].all() and ref["seq_flag"][honest].sum() == 2
        # TPR 3/3; at most floor(0.01 * 253) = 2 false positives, plus the honest sequence whose oracle mean IS the
        # threshold if the library's fp32 mean of it lands a rounding above (a near tie, excused and counted above)
        assert fl[stego].all() and fl[honest].sum() <= 2 + pooled_stats[name]["flag_excused"]
    _sampled_estimators(difr, wl, batch, g, deep, deep_host, host_args, say)
    del batch, g, i
    gc.collect()
    torch.cuda.empty_cache()
