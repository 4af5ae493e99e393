"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (one launch
over the whole resident batch).  The oracle cannot afford every row here, so it scores a seeded
sample (whole sequences plus scattered rows); all rows are covered by properties that hold at
any size.  Claims: the library's own samplers run on the prover logits (that is the workload),
except on the sampled rows, whose claims come from the oracle's samplers so that no oracle input
is produced by the HIP path."""
import gc
import sys

import numpy as np
import pytest
import torch

import oracle
import parity
from paper_2511_02620_amd import calibrate
from paper_2511_02620_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def f32(x):
    return float(np.float32(x))


@pytest.fixture(scope="module")
def difr():
    assert torch.cuda.is_available()
    import paper_2511_02620_amd as d

    d.load_library()
    return d


def _resident_batch(difr, wl, sample_rows):
    """Verifier logits for the whole workload in HBM, claims for both estimators, and the host copies
    (verifier and prover logits) of the sampled rows."""
    N, V = wl.N, wl.V
    T = wl.temperature
    logits = torch.empty(N, V, dtype=wl.dtype, device=DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    cg = torch.empty(N, dtype=torch.int32, device=DEV)
    ci = torch.empty(N, dtype=torch.int32, device=DEV)
    sample = torch.tensor(sample_rows, dtype=torch.int64)
    prov_host = np.empty((len(sample_rows), V), dtype=np.uint16)
    for c in range(wl.n_chunks):
        r0, r1 = c * wl.chunk_rows, (c + 1) * wl.chunk_rows
        ver, prov = wl.logits_chunk(c, DEV)
        logits[r0:r1] = ver
        cg[r0:r1] = difr.gumbel_score(prov, T, seeds, sid[r0:r1], pos[r0:r1], None, want_scores=False)["argmax"]
        ci[r0:r1] = difr.ipt_score(prov, T, seeds, sid[r0:r1], pos[r0:r1], None, want_token=True,
                                   want_interval=False)["ipt_token"]
        inside = torch.nonzero((sample >= r0) & (sample < r1)).flatten()
        if inside.numel():
            rows = (sample[inside] - r0).to(DEV)
            prov_host[inside.numpy()] = parity.to_host_logits(prov[rows])
        del ver, prov
    torch.cuda.synchronize()
    # honest claims of the sampled rows: the oracle's samplers on the prover logits
    hs = parity.seeds_u64(seeds)
    hsid = sid.cpu().numpy()[sample_rows]
    hpos = parity.positions_u32(pos)[sample_rows]
    og = oracle.gumbel_score(prov_host, V, f32(T), hs, hsid, hpos)["argmax"]
    oi = oracle.ipt_score(prov_host, V, f32(T), hs, hsid, hpos)["ipt_token"]
    hip_g, hip_i = cg[sample.to(DEV)].cpu().numpy(), ci[sample.to(DEV)].cpu().numpy()
    # the library's samplers agree with the oracle's except at near ties (a vocabulary of 150k entries has
    # many CDF intervals narrower than the tie width, so IPT near ties are not rare)
    gdiff, idiff = np.nonzero(hip_g != og)[0], np.nonzero(hip_i != oi)[0]
    say("sampler spot check on %d rows: gumbel differs on %d, ipt differs on %d" % (len(sample_rows), len(gdiff), len(idiff)))
    for k in gdiff:
        x = oracle.decode_row(prov_host[k])
        row = oracle.gumbel_row(x, f32(T), int(hs[hsid[k]]), int(hsid[k]), int(hpos[k]), int(hip_g[k]))
        assert row["margin"] < parity.TIE_REL * max(1.0, abs(row["max_score"])), "gumbel sampler differs beyond a near tie"
    for k in idiff:
        x = oracle.decode_row(prov_host[k])
        row = oracle.ipt_row(x, f32(T), int(hs[hsid[k]]), int(hsid[k]), int(hpos[k]), int(hip_i[k]))
        assert row["dist"] < parity.TIE_REL, "ipt sampler differs beyond a near tie"
    assert len(gdiff) <= 0.01 * len(sample_rows) and len(idiff) <= 0.02 * len(sample_rows)
    cg[sample.to(DEV)] = torch.from_numpy(og.copy()).to(DEV)
    ci[sample.to(DEV)] = torch.from_numpy(oi.copy()).to(DEV)
    del prov_host
    return logits, seeds, sid, pos, cg, ci


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


def _score_and_compare(difr, wl, logits, seeds, sid, pos, cg, ci, sample_rows, tau_g, tau_i):
    T = wl.temperature
    off = wl.seq_offsets().to(DEV)
    g = difr.gumbel_score(logits, T, seeds, sid, pos, cg)
    i = difr.ipt_score(logits, T, seeds, sid, pos, ci, want_log_mass=True)
    sg = difr.seq_reduce(g["margin"], g["flags"], off, tau_g)
    si = difr.seq_reduce(i["dist"], i["flags"], off, tau_i)
    g2 = difr.gumbel_score(logits, T, seeds, sid, pos, cg)           # same launch again: bit-identical
    i2 = difr.ipt_score(logits, T, seeds, sid, pos, ci, want_log_mass=True)
    torch.cuda.synchronize()
    for k in g:
        assert torch.equal(g[k], g2[k]), k
    for k in i:
        assert torch.equal(i[k], i2[k]), k
    del g2, i2
    # the one-pass call the benchmark times returns the same outputs, bit for bit, on every row
    gb, ib = difr.score_both(logits, T, seeds, sid, pos, cg, ci)
    torch.cuda.synchronize()
    for k in gb:
        assert torch.equal(torch.nan_to_num(gb[k], nan=-7.0) if gb[k].dtype.is_floating_point else gb[k],
                           torch.nan_to_num(g[k], nan=-7.0) if g[k].dtype.is_floating_point else g[k]), k
    for k in ib:
        assert torch.equal(torch.nan_to_num(ib[k], nan=-7.0) if ib[k].dtype.is_floating_point else ib[k],
                           torch.nan_to_num(i[k], nan=-7.0) if i[k].dtype.is_floating_point else i[k]), k
    del gb, ib
    _check_all_rows(g, i)
    # pooled means equal the fp64 mean of the row scores, for every sequence
    for scores, pooled in ((g["margin"], sg), (i["dist"], si)):
        want = scores.double().view(wl.S, wl.L).mean(dim=1)
        assert float((pooled["seq_mean"].double() - want).abs().max()) <= 1e-6 * max(1.0, float(want.abs().max()))
        assert torch.equal(pooled["seq_max"], scores.view(wl.S, wl.L).max(dim=1).values)
    # the oracle on the sampled rows
    sel = torch.tensor(sample_rows, dtype=torch.int64, device=DEV)
    host = parity.to_host_logits(logits[sel])
    hs = parity.seeds_u64(seeds)
    hsid, hpos = sid.cpu().numpy()[sample_rows], parity.positions_u32(pos)[sample_rows]
    og = oracle.gumbel_score(host, wl.V, f32(T), hs, hsid, hpos, cg[sel].cpu().numpy())
    oi = oracle.ipt_score(host, wl.V, f32(T), hs, hsid, hpos, ci[sel].cpu().numpy())
    st_g = parity.compare_gumbel({k: v[sel] for k, v in g.items()}, og)
    st_i = parity.compare_ipt({k: v[sel] for k, v in i.items()}, oi, host, wl.V, (f32(T), hs, hsid, hpos), 0.01)
    say(wl.name, "T=%g" % T, "gumbel", st_g)
    say(wl.name, "T=%g" % T, "ipt", st_i)
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
    say(wl.name, "T=%g" % T, "admissible set at delta 2.5: mean size %.2f over all rows, %d near-threshold sampled rows"
        % (float(a2["count"].float().mean()), int((~sure).sum())))
    # the same count from the one-pass call, with both scores: every row determined and equal to the two-pass count
    g1, i1, a3 = difr.score_both_admissible(logits, T, seeds, sid, pos, 2.5, cg, ci)
    torch.cuda.synchronize()
    assert torch.equal(a3["count"], a2["count"]), int((a3["count"] != a2["count"]).sum())
    for k in g1:
        assert torch.equal(torch.nan_to_num(g1[k].float(), nan=-7.0), torch.nan_to_num(g[k].float(), nan=-7.0)), k
    for k in i1:
        ref = i[k] & 0xF7 if k == "flags" else i[k]      # the honest-token search of difr_ipt_score sets SLOW_PATH
        assert torch.equal(torch.nan_to_num(i1[k].float(), nan=-7.0), torch.nan_to_num(ref.float(), nan=-7.0)), k
    # Token-DiFR likelihood estimate with the paper's generation policy (top-k 50, top-p 0.95) on every row;
    # the oracle on the first 384 sampled rows (it sorts the whole vocabulary twice per row)
    z = torch.randn(256, generator=torch.Generator().manual_seed(5), dtype=torch.float32)
    lk = difr.gumbel_likelihood(logits, T, seeds, sid, pos, cg, z.to(DEV), top_k=50, top_p=0.95, s=16, sigma=0.3,
                                want_active=True)
    torch.cuda.synchronize()
    pi_all = lk["pi"]
    assert ((pi_all >= 0) & (pi_all <= 1)).all() and (lk["flags"] == 0).all()
    sub = sample_rows[:384]
    ssel = torch.tensor(sub, dtype=torch.int64, device=DEV)
    ol = oracle.likelihood(host[:384], wl.V, f32(T), hs, hsid[:384], hpos[:384], cg[ssel].cpu().numpy(), 50,
                           float(f32(0.95)), 16, float(f32(0.3)), z.double().numpy())
    assert np.array_equal(lk["tau"][ssel].cpu().numpy(), ol["tau"].astype(np.float32))
    diff = (lk["active"][ssel].cpu().numpy() != ol["active"]).any(axis=1)
    excused = diff & (ol["gap_s"] < 1e-5)
    assert not (diff & ~excused).any()
    perr = np.where(excused, 0.0, np.abs(lk["pi"][ssel].cpu().numpy().astype(np.float64) - ol["pi"]))
    assert perr.max() <= 1e-4
    # Token-IPT-DiFR under the same filter, every row; the oracle on the same 384 rows
    fi = difr.ipt_score_filtered(logits, T, seeds, sid, pos, ci, top_k=50, top_p=0.95)
    torch.cuda.synchronize()
    assert ((fi["dist"] >= 0) & (fi["dist"] < 1)).all() and (fi["flags"] & 6 == 0).all() and (fi["kept"] >= 1).all()
    ofi = oracle.ipt_filtered_score(host[:384], wl.V, f32(T), hs, hsid[:384], hpos[:384], ci[ssel].cpu().numpy(), 50,
                                    float(f32(0.95)))
    assert np.array_equal(fi["kept"][ssel].cpu().numpy(), ofi["kept"])
    st_f = parity.compare_ipt({k: v[ssel] for k, v in fi.items() if k != "kept"}, ofi)
    say(wl.name, "T=%g" % T, "filtered ipt:", st_f, "mean kept %.1f" % float(fi["kept"].float().mean()))
    # the two filtered estimators from one read of the logits: identical to the two calls on every row
    lk2, fi2 = difr.score_both_filtered(logits, T, seeds, sid, pos, cg, ci, z.to(DEV), top_k=50, top_p=0.95, s=16,
                                        sigma=0.3, want_active=True)
    torch.cuda.synchronize()
    for name, a_, b_ in (("likelihood", lk, lk2), ("filtered ipt", fi, fi2)):
        for k in a_:
            assert torch.equal(torch.nan_to_num(a_[k].float(), nan=-7.0), torch.nan_to_num(b_[k].float(), nan=-7.0)), (name, k)
    del lk2, fi2
    # the bare nucleus (no top-k): every row, the oracle on the first 128 sampled rows at top_p and top_p -/+ 2e-6
    # (the kept-set size of a nucleus of tens of thousands of tokens is decided by fp32 masses)
    nu = difr.ipt_score_filtered(logits, T, seeds, sid, pos, ci, top_k=0, top_p=0.9)
    torch.cuda.synchronize()
    assert (nu["kept"] >= 1).all() and (nu["flags"] & 6 == 0).all()
    nsel = ssel[:128]
    onu = [oracle.ipt_filtered_score(host[:128], wl.V, f32(T), hs, hsid[:128], hpos[:128], ci[nsel].cpu().numpy(), 0,
                                     float(f32(0.9)) + dp) for dp in (0.0, -2e-6, 2e-6)]
    kn = nu["kept"][nsel].cpu().numpy()
    assert (kn >= onu[1]["kept"]).all() and (kn <= onu[2]["kept"]).all()
    for name in ("cdf_lo", "cdf_hi", "dist"):
        assert np.abs(nu[name][nsel].cpu().numpy().astype(np.float64) - onu[0][name]).max() <= 1e-4, name
    say(wl.name, "T=%g" % T, "nucleus 0.9: mean kept %.0f over all rows; %d of 128 oracle rows with the same size"
        % (float(nu["kept"].float().mean()), int((kn == onu[0]["kept"]).sum())))
    say(wl.name, "T=%g" % T, "likelihood: mean pi %.4f over all rows, worst error %.3g on %d oracle rows, %d excused"
        % (float(pi_all.mean()), perr.max(), len(sub), int(excused.sum())))
    return g, i, sg, si, og, oi, st_g, st_i


def _whole_sequence_pooling(wl, seqs, sample_rows, og, oi, sg, si, tau_g, tau_i, st_g, st_i):
    """Oracle pooling over the whole sequences that are inside the sample."""
    index = {r: k for k, r in enumerate(sample_rows)}
    for s in seqs:
        ks = [index[s * wl.L + j] for j in range(wl.L)]
        for o, pooled, tau, key, st in ((og, sg, tau_g, "margin", st_g), (oi, si, tau_i, "dist", st_i)):
            ref = oracle.seq_reduce(o[key][ks], o["flags"][ks], np.array([0, wl.L]), np.float32(tau))
            got = {k: v[s:s + 1] for k, v in pooled.items()}
            parity.compare_seq(got, ref, float(tau), st["match_excused"])


@pytest.mark.parametrize("T", [1.0, 0.6])
def test_c3_full_size(difr, T):
    wl = W.C3_30B.with_temperature(T)
    rng = np.random.default_rng(31 + int(T * 10))
    seqs = [0, 37]
    sample_rows = sorted(set([s * wl.L + j for s in seqs for j in range(wl.L)])
                         | set(int(r) for r in rng.integers(0, wl.N, size=512)) | {wl.N - 1})
    batch = _resident_batch(difr, wl, sample_rows)
    tau_g, tau_i = 0.02, 0.001
    g, i, sg, si, og, oi, st_g, st_i = _score_and_compare(difr, wl, *batch, sample_rows, tau_g, tau_i)
    _whole_sequence_pooling(wl, seqs, sample_rows, og, oi, sg, si, tau_g, tau_i, st_g, st_i)
    match = float((g["flags"] & 1).float().mean())
    say("C3 T=%g gumbel match rate %.4f" % (T, match))
    assert match > 0.98                                 # bf16-level drift flips well under 2% of the samples
    del batch, g, i
    gc.collect()
    torch.cuda.empty_cache()


def test_c5_stego_audit_full_size(difr):
    wl = W.C5_STEGO
    stego = wl.stego_sequences()
    assert len(stego) == 3
    honest = [s for s in range(wl.S) if s not in stego]
    seqs = stego + honest[:5]
    sample_rows = sorted(s * wl.L + j for s in seqs for j in range(wl.L))
    logits, seeds, sid, pos, cg, ci = _resident_batch(difr, wl, sample_rows)
    # the stego recipe overwrites the claims of the stego sequences (both estimators)
    for c in range(wl.n_chunks):
        r0, r1 = c * wl.chunk_rows, (c + 1) * wl.chunk_rows
        if any(r0 < (s + 1) * wl.L and r1 > s * wl.L for s in stego):
            cg[r0:r1] = wl.mutate_claims(c, cg[r0:r1], logits[r0:r1])
            ci[r0:r1] = wl.mutate_claims(c, ci[r0:r1], logits[r0:r1])
    # the deployment calibrates on its own benign traffic: thresholds from the library's pooled means
    off = wl.seq_offsets().to(DEV)
    T = wl.temperature
    m_g = difr.seq_reduce(difr.gumbel_score(logits, T, seeds, sid, pos, cg)["margin"], None, off, 0.0)["seq_mean"].cpu().numpy()
    m_i = difr.seq_reduce(difr.ipt_score(logits, T, seeds, sid, pos, ci)["dist"], None, off, 0.0)["seq_mean"].cpu().numpy()
    tau_g = calibrate.threshold_for_fpr(m_g[honest], 1e-2)
    tau_i = calibrate.threshold_for_fpr(m_i[honest], 1e-2)
    g, i, sg, si, og, oi, st_g, st_i = _score_and_compare(difr, wl, logits, seeds, sid, pos, cg, ci, sample_rows, tau_g, tau_i)
    _whole_sequence_pooling(wl, seqs, sample_rows, og, oi, sg, si, tau_g, tau_i, st_g, st_i)
    for name, pooled, tau in (("margin", sg, tau_g), ("dist", si, tau_i)):
        fl = pooled["seq_flag"].cpu().numpy()
        mean = pooled["seq_mean"].cpu().numpy()
        say("C5", name, "tau %.5g" % tau, "stego means", mean[stego], "flagged", fl[stego].tolist(),
            "honest flagged", int(fl[honest].sum()), "honest mean of means %.5g" % mean[honest].mean())
        assert np.array_equal(fl, (~(mean <= np.float32(tau))).astype(np.uint8))
        assert fl[stego].all() and fl[honest].sum() <= 2            # TPR 3/3, at most floor(0.01 * 253) false positives
    del logits, g, i
    gc.collect()
    torch.cuda.empty_cache()
