"""GPU parity: the HIP library, called through its C ABI (ctypes binding), against the CPU
oracle on identical seeded inputs.  Every test here needs a real MI355X."""
import math
import sys

import numpy as np
import pytest
import torch

import oracle
import parity
from paper_2511_02620_amd import workloads as W

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def difr():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2511_02620_amd as d

    d.load_library()
    return d


DEV = "cuda:0"


def f32(x):
    """The temperature argument of the C ABI is a float: the oracle gets the same fp32 value."""
    return float(np.float32(x))


def u32_as_i32(t):
    t = t.to(torch.int64) % (1 << 32)
    return torch.where(t >= (1 << 31), t - (1 << 32), t).to(torch.int32)


def _aux(wl, dev=DEV):
    return (wl.seeds().to(dev), wl.seq_ids().to(dev), wl.positions().to(dev), wl.seq_offsets().to(dev))


def _oracle_claims(wl, prover_host, row0):
    """Honest claims of rows [row0, row0+R): the oracle samplers run on the prover logits."""
    R = prover_host.shape[0]
    seeds = parity.seeds_u64(wl.seeds())
    sid = wl.seq_ids().numpy()[row0:row0 + R]
    pos = parity.positions_u32(wl.positions())[row0:row0 + R]
    g = oracle.gumbel_score(prover_host, wl.V, f32(wl.temperature), seeds, sid, pos)["argmax"]
    i = oracle.ipt_score(prover_host, wl.V, f32(wl.temperature), seeds, sid, pos)["ipt_token"]
    return torch.from_numpy(g.copy()), torch.from_numpy(i.copy())


def _build_small(wl):
    """Whole workload on the GPU plus oracle-made claims (small workloads only)."""
    ver, cg, ci = [], [], []
    for c in range(wl.n_chunks):
        v, p = wl.logits_chunk(c, DEV)
        hg, hi = _oracle_claims(wl, parity.to_host_logits(p), c * wl.chunk_rows)
        cg.append(wl.mutate_claims(c, hg, v))
        ci.append(wl.mutate_claims(c, hi, v))
        ver.append(v)
        del p
    return torch.cat(ver), torch.cat(cg).to(DEV), torch.cat(ci).to(DEV)


def _score_both_ways(difr, wl, logits, claims_g, claims_i, sigma=0.01, eps=1e-30, temps=None):
    seeds, sid, pos, _ = _aux(wl)
    host = parity.to_host_logits(logits)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    ht = None if temps is None else temps.cpu().numpy()
    gg = difr.gumbel_score(logits, wl.temperature, seeds, sid, pos, claims_g, temperatures=temps, V=wl.V)
    gi = difr.ipt_score(logits, wl.temperature, seeds, sid, pos, claims_i, temperatures=temps, V=wl.V,
                        want_token=True, want_log_mass=True, sigma=sigma, eps=eps)
    torch.cuda.synchronize()
    og = oracle.gumbel_score(host, wl.V, f32(wl.temperature), hs, hsid, hpos, claims_g.cpu().numpy(), ht)
    oi = oracle.ipt_score(host, wl.V, f32(wl.temperature), hs, hsid, hpos, claims_i.cpu().numpy(), ht, sigma, eps)
    sg = parity.compare_gumbel(gg, og)
    si = parity.compare_ipt(gi, oi, host, wl.V, (f32(wl.temperature) if ht is None else ht, hs, hsid, hpos), sigma)
    return gg, gi, og, oi, sg, si


def test_noise_bits_bit_exact(difr):
    wl = W.scaled(W.C3_30B, S=3, L=4, chunk_rows=12)
    seeds, sid, pos, _ = _aux(wl)
    logits = torch.zeros(wl.N, wl.V, dtype=torch.bfloat16, device=DEV)
    hs = parity.seeds_u64(seeds)
    for row in (0, 5, 11):
        for stream in (0, 1):
            bits = difr.debug_noise(logits, 1.0, seeds, sid, pos, row, stream).cpu().numpy().view(np.uint32)
            s = int(sid[row])
            want = oracle.noise_row(int(hs[s]), s, int(pos[row]), stream, wl.V)
            assert np.array_equal(bits, want), (row, stream)
    # ragged vocabulary: the last Philox block is partial
    wl2 = W.scaled(W.C1_TINY, S=1, L=1, V=1023, chunk_rows=1)
    seeds, sid, pos, _ = _aux(wl2)
    bits = difr.debug_noise(torch.zeros(1, 1023, device=DEV), 1.0, seeds, sid, pos, 0, 0).cpu().numpy().view(np.uint32)
    assert np.array_equal(bits, oracle.noise_row(int(parity.seeds_u64(seeds)[0]), 0, 0, 0, 1023))
    # host helper agrees with the oracle block function
    assert difr.philox4x32_10([1, 2, 3, 4], [5, 6]) == [int(x) for x in oracle.philox4x32_10([1, 2, 3, 4], [5, 6])]


def test_gumbel_map_exhaustive(difr):
    """Every one of the 2^23 uniforms: device fp32 g against the oracle's double."""
    k = torch.arange(1 << 23, dtype=torch.int64, device=DEV)
    bits = u32_as_i32(k << 9)
    g = difr.debug_gumbel_map(bits).cpu().numpy().astype(np.float64)
    want = oracle.gumbel_from_bits(np.arange(1 << 23, dtype=np.uint32) << np.uint32(9))
    err = np.abs(g - want)
    say("gumbel map: max abs err %.3g at k=%d" % (err.max(), int(err.argmax())))
    assert err.max() <= 4e-6
    # low 9 bits of the word are not used
    g2 = difr.debug_gumbel_map(bits[:4096] | 0x1FF).cpu().numpy()
    assert np.array_equal(g2.astype(np.float64), g[:4096])


def test_c1_tiny_every_row(difr):
    wl = W.C1_TINY
    logits, cg, ci = _build_small(wl)
    gg, gi, og, oi, sg, si = _score_both_ways(difr, wl, logits, cg, ci)
    say("C1 gumbel", sg)
    say("C1 ipt", si)
    # about 90% of the claims are honest (drift 1e-3 rarely flips the sample)
    assert 0.75 < (og["flags"] & 1).mean() <= 1.0 and 0.75 < (oi["flags"] & 1).mean() <= 1.0
    for name, scores_g, scores_o, fl_g, fl_o, excused in (("margin", gg["margin"], og["margin"], gg["flags"], og["flags"], sg["match_excused"]),
                                                          ("dist", gi["dist"], oi["dist"], gi["flags"], oi["flags"], si["match_excused"])):
        tau = 0.05
        off = wl.seq_offsets()
        gs = difr.seq_reduce(scores_g, fl_g, off.to(DEV), tau)
        os_ = oracle.seq_reduce(scores_o, fl_o, off.numpy(), tau)
        say("C1 pool", name, parity.compare_seq(gs, os_, tau, excused))


def test_honest_claims_identical_logits_margin_zero(difr):
    """Scoring the sampler's own output on the same logits gives margin exactly 0 / dist exactly 0."""
    wl = W.scaled(W.C2_3B, S=4, L=32, V=4104, chunk_rows=128)
    v, _ = wl.logits_chunk(0, DEV)
    seeds, sid, pos, _ = _aux(wl)
    samp = difr.gumbel_score(v, wl.temperature, seeds, sid, pos)
    assert ((samp["flags"] & 2) != 0).all() and torch.isnan(samp["margin"]).all()
    again = difr.gumbel_score(v, wl.temperature, seeds, sid, pos, samp["argmax"])
    assert (again["margin"] == 0).all() and ((again["flags"] & 1) == 1).all()
    isamp = difr.ipt_score(v, wl.temperature, seeds, sid, pos, want_token=True)
    iagain = difr.ipt_score(v, wl.temperature, seeds, sid, pos, isamp["ipt_token"], want_token=True)
    assert (iagain["dist"] == 0).all()
    # MATCH is the half-open test; the sampler's token can only miss it when u sits on an edge in fp32
    assert ((iagain["flags"] & 1) == 1).float().mean() > 0.99
    assert (iagain["ipt_token"] == isamp["ipt_token"]).float().mean() > 0.99


def test_c2_3b_class_every_row(difr):
    wl = W.C2_3B
    logits, cg, ci = _build_small(wl)
    gg, gi, og, oi, sg, si = _score_both_ways(difr, wl, logits, cg, ci)
    say("C2 gumbel", sg)
    say("C2 ipt", si)
    mism_g = 1.0 - (og["flags"] & 1).mean()
    mism_i = 1.0 - (oi["flags"] & 1).mean()
    say("C2 oracle mismatch rates: gumbel %.4f ipt %.4f" % (mism_g, mism_i))
    assert 0.005 < mism_g < 0.08 and 0.005 < mism_i < 0.08       # ~2% swapped + benign drift flips
    tau = 0.02
    off = wl.seq_offsets()
    gs = difr.seq_reduce(gg["margin"], gg["flags"], off.to(DEV), tau)
    say("C2 pool margin", parity.compare_seq(gs, oracle.seq_reduce(og["margin"], og["flags"], off.numpy(), tau), tau,
                                             sg["match_excused"]))
    gs = difr.seq_reduce(gi["dist"], gi["flags"], off.to(DEV), tau)
    say("C2 pool dist", parity.compare_seq(gs, oracle.seq_reduce(oi["dist"], oi["flags"], off.numpy(), tau), tau,
                                           si["match_excused"]))


@pytest.mark.parametrize("dtype,V,ld,offset", [
    (torch.bfloat16, 1, 8, 0), (torch.bfloat16, 7, 7, 0), (torch.bfloat16, 1000, 1000, 0),
    (torch.bfloat16, 2055, 2064, 0), (torch.bfloat16, 4099, 4099, 1), (torch.bfloat16, 8192, 8200, 3),
    (torch.float32, 1, 1, 0), (torch.float32, 5, 8, 0), (torch.float32, 1023, 1023, 0),
    (torch.float32, 4100, 4104, 0), (torch.float32, 3001, 3001, 1),
])
def test_ragged_shapes_and_unaligned_rows(difr, dtype, V, ld, offset):
    """Vocabulary sizes that are not a multiple of the vector width, padded pitches whose padding
    holds garbage, and rows that are not 16-byte aligned (generic load path)."""
    N = 37
    g = torch.Generator(device=DEV).manual_seed(1234 + V)
    store = torch.randn(N * ld + offset + 8, generator=g, device=DEV, dtype=torch.float32).mul_(2.5).to(dtype)
    logits = store[offset:offset + N * ld].view(N, ld)
    if ld > V:
        logits[:, V:] = float("nan")                                # padding must never be read as data
    wl = W.scaled(W.C1_TINY, S=3, L=13, V=V, chunk_rows=39)
    seeds = wl.seeds().to(DEV)
    sid = wl.seq_ids()[:N].to(DEV)
    pos = u32_as_i32(wl.positions()[:N].to(torch.int64) * 1000003 + 4000000000).to(DEV)   # large uint32 positions
    claims = torch.randint(0, V, (N,), generator=torch.Generator().manual_seed(V), dtype=torch.int32).to(DEV)
    host = parity.to_host_logits(logits)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    gg = difr.gumbel_score(logits, 0.9, seeds, sid, pos, claims, V=V)
    gi = difr.ipt_score(logits, 0.9, seeds, sid, pos, claims, V=V, want_token=True, want_log_mass=True)
    og = oracle.gumbel_score(host, V, np.float32(0.9), hs, hsid, hpos, claims.cpu().numpy())
    oi = oracle.ipt_score(host, V, np.float32(0.9), hs, hsid, hpos, claims.cpu().numpy())
    parity.compare_gumbel(gg, og)
    parity.compare_ipt(gi, oi, host, V, (np.float32(0.9), hs, hsid, hpos), 0.01)


def test_row_level_conditions(difr):
    """Invalid claims, masked (-inf) entries, NaN / +inf logits, per-row temperatures, bad sequence ids."""
    N, V = 24, 3000
    g = torch.Generator(device=DEV).manual_seed(99)
    logits = torch.randn(N, V, generator=g, device=DEV).mul_(2).to(torch.bfloat16)
    logits[3, 100:2900] = float("-inf")             # heavily masked row
    logits[4, :] = float("-inf")
    logits[4, 17] = 1.0                              # one live entry
    logits[5, 7] = float("nan")
    logits[6, 2999] = float("inf")
    wl = W.scaled(W.C1_TINY, S=4, L=6, V=V, chunk_rows=24)
    seeds, sid, pos, _ = _aux(wl)
    claims = torch.randint(0, V, (N,), generator=torch.Generator().manual_seed(5), dtype=torch.int32)
    claims[0] = -1
    claims[1] = V
    claims[4] = 17
    claims[3] = 150                                  # a masked token is claimed
    claims = claims.to(DEV)
    temps = torch.linspace(0.5, 1.6, N).to(DEV)
    host = parity.to_host_logits(logits)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    gg = difr.gumbel_score(logits, 1.0, seeds, sid, pos, claims, temperatures=temps)
    gi = difr.ipt_score(logits, 1.0, seeds, sid, pos, claims, temperatures=temps, want_token=True, want_log_mass=True)
    og = oracle.gumbel_score(host, V, 1.0, hs, hsid, hpos, claims.cpu().numpy(), temps.cpu().numpy())
    oi = oracle.ipt_score(host, V, 1.0, hs, hsid, hpos, claims.cpu().numpy(), temps.cpu().numpy())
    ok = np.ones(N, bool)
    ok[[5, 6]] = False                               # outputs unspecified on non-finite rows, flag only
    fg, fi = gg["flags"].cpu().numpy(), gi["flags"].cpu().numpy()
    assert fg[5] & 4 and fg[6] & 4 and fi[5] & 4 and fi[6] & 4
    assert not (fg[ok] & 4).any() and not (fi[ok] & 4).any()
    sel = torch.from_numpy(np.nonzero(ok)[0]).to(DEV)
    parity.compare_gumbel({k: v[sel] for k, v in gg.items()}, {k: v[ok] for k, v in og.items()})
    parity.compare_ipt({k: v[sel] for k, v in gi.items()}, {k: v[ok] for k, v in oi.items()}, host[ok], V,
                       (temps.cpu().numpy()[ok], hs, hsid[ok], hpos[ok]), 0.01)
    assert fg[0] & 2 and fg[1] & 2 and math.isnan(float(gg["margin"][0])) and int(gg["argmax"][0]) == int(og["argmax"][0])
    assert int(gg["argmax"][4]) == 17 and float(gg["margin"][4]) == 0.0 and float(gi["dist"][4]) == 0.0
    # a bad temperature or sequence id poisons only its own row
    temps2 = temps.clone()
    temps2[2] = 0.0
    temps2[7] = float("nan")
    sid2 = sid.clone()
    sid2[9] = 4
    sid2[10] = -1
    g2 = difr.gumbel_score(logits, 1.0, seeds, sid2, pos, claims, temperatures=temps2)
    i2 = difr.ipt_score(logits, 1.0, seeds, sid2, pos, claims, temperatures=temps2)
    for out in (g2, i2):
        f = out["flags"].cpu().numpy()
        assert f[2] & 4 and f[7] & 4 and f[9] & 2 and f[10] & 2
    keep = [r for r in range(N) if r not in (2, 7, 9, 10, 5, 6)]
    same = lambda a, b: torch.equal(torch.nan_to_num(a[keep], nan=-7.0), torch.nan_to_num(b[keep], nan=-7.0))
    assert same(g2["margin"], gg["margin"]) and same(i2["dist"], gi["dist"])


def test_empty_batch_and_determinism(difr):
    wl = W.scaled(W.C2_3B, S=2, L=64, V=20000, chunk_rows=128)
    v, _ = wl.logits_chunk(0, DEV)
    seeds, sid, pos, off = _aux(wl)
    empty = difr.gumbel_score(v[:0], 1.0, seeds, sid[:0], pos[:0], None, V=wl.V)
    assert empty["margin"].numel() == 0
    assert difr.ipt_score(v[:0], 1.0, seeds, sid[:0], pos[:0], None, V=wl.V)["dist"].numel() == 0
    claims = torch.randint(0, wl.V, (wl.N,), dtype=torch.int32).to(DEV)
    a = difr.gumbel_score(v, 0.7, seeds, sid, pos, claims)
    b = difr.gumbel_score(v, 0.7, seeds, sid, pos, claims)
    for k in a:
        assert torch.equal(a[k], b[k]), k
    a = difr.ipt_score(v, 0.7, seeds, sid, pos, claims, want_token=True, want_log_mass=True)
    b = difr.ipt_score(v, 0.7, seeds, sid, pos, claims, want_token=True, want_log_mass=True)
    for k in a:
        assert torch.equal(a[k], b[k]), k
    # a non-default stream gives the same answer
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        c = difr.gumbel_score(v, 0.7, seeds, sid, pos, claims)
    s.synchronize()
    ref = difr.gumbel_score(v, 0.7, seeds, sid, pos, claims)
    assert torch.equal(c["margin"], ref["margin"]) and torch.equal(c["argmax"], ref["argmax"])


def test_seq_reduce_ragged(difr):
    rng = np.random.default_rng(3)
    lens = [0, 1, 255, 256, 257, 1024, 0, 3000, 5]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    N = int(off[-1])
    scores = rng.exponential(0.2, size=N).astype(np.float32)
    flags = (rng.uniform(size=N) < 0.9).astype(np.uint8)
    tau = 0.2
    gs = difr.seq_reduce(torch.from_numpy(scores).to(DEV), torch.from_numpy(flags).to(DEV), torch.from_numpy(off).to(DEV), tau)
    os_ = oracle.seq_reduce(scores.astype(np.float64), flags, off, np.float32(tau))
    say("seq_reduce ragged", parity.compare_seq(gs, os_, tau))
    assert list(gs["seq_flag"].cpu().numpy()[[0, 6]]) == [0, 0]
    scores[600] = np.nan                                             # inside sequence 4
    gs = difr.seq_reduce(torch.from_numpy(scores).to(DEV), None, torch.from_numpy(off).to(DEV), tau)
    os_ = oracle.seq_reduce(scores.astype(np.float64), None, off, np.float32(tau))
    parity.compare_seq(gs, os_, tau)
    assert int(gs["seq_flag"][4]) == 1 and math.isnan(float(gs["seq_mean"][4])) and math.isnan(float(gs["seq_max"][4]))
    assert difr.seq_reduce(torch.zeros(0, device=DEV), None, torch.zeros(1, dtype=torch.int64, device=DEV), 0.0)["seq_mean"].numel() == 0


def test_c5_stego_audit_scaled(difr):
    """The stego-audit recipe at a vocabulary the oracle can afford for every row: stego sequences pick among
    their top-4 tokens, per-sequence means, threshold calibrated on the oracle's honest means at FPR 1e-2."""
    wl = W.scaled(W.C5_STEGO, S=256, L=32, V=8200, chunk_rows=512)
    logits, cg, ci = _build_small(wl)
    gg, gi, og, oi, sg, si = _score_both_ways(difr, wl, logits, cg, ci)
    say("C5s gumbel", sg)
    say("C5s ipt", si)
    off = wl.seq_offsets()
    stego = wl.stego_sequences()
    honest = np.array([s for s in range(wl.S) if s not in stego])
    assert len(stego) == 3
    for name, sc_g, sc_o, fl_g, fl_o, exc in (("margin", gg["margin"], og["margin"], gg["flags"], og["flags"], sg["match_excused"]),
                                              ("dist", gi["dist"], oi["dist"], gi["flags"], oi["flags"], si["match_excused"])):
        means = oracle.seq_reduce(sc_o, fl_o, off.numpy(), 0.0)["seq_mean"]
        tau = np.float32(oracle.calibrate_threshold(means[honest], 1e-2))
        os_ = oracle.seq_reduce(sc_o, fl_o, off.numpy(), tau)
        gs = difr.seq_reduce(sc_g, fl_g, off.to(DEV), float(tau))
        st = parity.compare_seq(gs, os_, float(tau), exc)
        flags = gs["seq_flag"].cpu().numpy()
        say("C5s pool", name, st, "tau %.5g" % tau, "stego flagged", flags[stego].tolist(), "honest flagged", int(flags[honest].sum()))
        assert flags[stego].all() and os_["seq_flag"][stego].all()      # every stego sequence is caught
        assert os_["seq_flag"][honest].sum() <= 2                       # floor(0.01 * 253), by construction of tau
        assert flags[honest].sum() <= 2 + st["flag_excused"]            # the sequence tau was read from may tip over


def _same_outputs(a, b):
    for k in a:
        x, y = a[k], b[k]
        if x.dtype.is_floating_point:
            assert torch.equal(torch.nan_to_num(x, nan=-7.0), torch.nan_to_num(y, nan=-7.0)), k
        else:
            assert torch.equal(x, y), k


@pytest.mark.parametrize("case", ["honest", "random_claims", "sampling", "peaked", "positive_offset", "small_offset",
                                  "masked_topk",
                                  "per_row_T", "fp32", "adversarial_order", "nonfinite"])
def test_filtered_kernel_equals_unfiltered_bit_for_bit(difr, case):
    """The exact pre-filter only skips entries that cannot reach the row maximum: every output of
    difr_gumbel_score must equal the unfiltered kernel's bit for bit, whatever the claims and logits."""
    wl = W.scaled(W.C3_30B, S=8, L=32, V=20504, chunk_rows=256)          # 2563 vectors: 10 full rounds + a partial one
    v, p = wl.logits_chunk(0, DEV)
    seeds, sid, pos, _ = _aux(wl)
    T = 0.8
    temps = None
    honest = difr.gumbel_score(p, T, seeds, sid, pos, unfiltered=True)["argmax"]
    claims = honest
    g = torch.Generator().manual_seed(77)
    if case == "random_claims":
        claims = torch.randint(0, wl.V, (wl.N,), generator=g, dtype=torch.int32).to(DEV)
    elif case == "sampling":
        claims = None
    elif case == "peaked":                       # one dominant logit per row: positive logit gate
        idx = torch.randint(0, wl.V, (wl.N,), generator=g).to(DEV)
        v = v.clone()
        v[torch.arange(wl.N, device=DEV), idx] = 25.0
        claims = torch.where(torch.arange(wl.N, device=DEV) % 3 == 0, honest, idx.to(torch.int32))
    elif case == "positive_offset":              # softmax is shift invariant, real logits sit anywhere
        v = (v.float() + 40.0).to(torch.bfloat16)
    elif case == "small_offset":                 # row maximum between the two noise bounds: logit caps of both signs
        v = (v.float() + 4.0).to(torch.bfloat16)
        claims = difr.gumbel_score(v, T, seeds, sid, pos, unfiltered=True)["argmax"]
    elif case == "masked_topk":                  # caller-side top-50 filter: everything else is -inf
        kth = v.float().topk(50, dim=1).values[:, -1:]
        v = torch.where(v.float() >= kth, v, torch.full_like(v, float("-inf")))
        claims = difr.gumbel_score(v, T, seeds, sid, pos, unfiltered=True)["argmax"]
    elif case == "per_row_T":
        temps = torch.linspace(0.3, 2.5, wl.N).to(DEV)
    elif case == "fp32":
        v = v.float() * 1.7
    elif case == "adversarial_order":            # ascending logits: the running bound keeps rising
        v = v.float().sort(dim=1).values.to(torch.bfloat16)
        claims = torch.zeros(wl.N, dtype=torch.int32, device=DEV)
    elif case == "nonfinite":
        v = v.clone()
        v[3, 1000] = float("nan")
        v[5, 20503] = float("inf")
        v[7, 0] = float("inf")
    a = difr.gumbel_score(v, T, seeds, sid, pos, claims, temperatures=temps)
    b = difr.gumbel_score(v, T, seeds, sid, pos, claims, temperatures=temps, unfiltered=True)
    torch.cuda.synchronize()
    if case == "nonfinite":
        fa, fb = a["flags"].cpu().numpy(), b["flags"].cpu().numpy()
        assert (fa[[3, 5, 7]] & 4).all() and (fb[[3, 5, 7]] & 4).all()
        keep = torch.tensor([r for r in range(wl.N) if r not in (3, 5, 7)], device=DEV)
        a = {k: x[keep] for k, x in a.items()}
        b = {k: x[keep] for k, x in b.items()}
    _same_outputs(a, b)
    if case in ("honest", "positive_offset", "fp32"):
        say(case, "match rate", float((a["flags"] & 1).float().mean()))


@pytest.mark.parametrize("dtype,V,ld,offset,case", [
    (torch.bfloat16, 20504, 20504, 0, "honest"),      # 10 full rounds + a partial one
    (torch.bfloat16, 20504, 20504, 0, "mutated"),
    (torch.bfloat16, 20504, 20504, 0, "sampling"),
    (torch.bfloat16, 20504, 20504, 0, "invalid"),
    (torch.bfloat16, 20504, 20504, 0, "small_offset"),
    (torch.bfloat16, 16384, 16384, 0, "mutated"),     # full rounds only
    (torch.bfloat16, 2051, 2056, 0, "mutated"),       # ragged last vector
    (torch.bfloat16, 300, 304, 0, "mutated"),         # less than one round
    (torch.float32, 4100, 4100, 0, "mutated"),
    (torch.float32, 5003, 5004, 0, "honest"),
    (torch.bfloat16, 4099, 4099, 1, "mutated"),       # unaligned rows: the two generic kernels
])
def test_score_both_equals_the_two_single_calls(difr, dtype, V, ld, offset, case):
    """difr_score_both shares one read of the row between the two estimators; every output must equal
    what difr_gumbel_score and difr_ipt_score return for the same claims, bit for bit."""
    N = 96
    g = torch.Generator().manual_seed(1234 + V)
    store = torch.empty(N * ld + offset + 8, dtype=dtype, device=DEV)
    x = (torch.randn(N, V, generator=g) * 2.5 + (4.0 if case == "small_offset" else 0.0)).to(dtype)
    logits = store[offset:offset + N * ld].view(N, ld)
    logits[:, :V] = x.to(DEV)
    seeds = torch.tensor([0x1234ABCD00000077, 5, -1], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 3).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    T = 0.7
    temps = torch.linspace(0.4, 1.6, N).to(DEV) if case == "small_offset" else None
    cg = difr.gumbel_score(logits, T, seeds, sid, pos, V=V, temperatures=temps)["argmax"]
    ci = difr.ipt_score(logits, T, seeds, sid, pos, V=V, temperatures=temps, want_token=True)["ipt_token"]
    if case == "mutated":                      # a third of the claims replaced, independently per estimator
        r1 = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
        r2 = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
        k = torch.arange(N, device=DEV)
        cg = torch.where(k % 3 == 1, r1, cg)
        ci = torch.where(k % 3 == 2, r2, ci)
    elif case == "invalid":
        cg = cg.clone(); ci = ci.clone()
        cg[::5] = -1; ci[1::5] = V; cg[2::5] = V + 3
    elif case == "sampling":
        cg = ci = None
    a = difr.gumbel_score(logits, T, seeds, sid, pos, cg, V=V, temperatures=temps)
    b = difr.ipt_score(logits, T, seeds, sid, pos, ci, V=V, temperatures=temps, want_interval=True)
    fa, fb = difr.score_both(logits, T, seeds, sid, pos, cg, ci, V=V, temperatures=temps)
    torch.cuda.synchronize()
    _same_outputs(fa, {k: a[k] for k in fa})
    _same_outputs(fb, {k: b[k] for k in fb})
    # the same with the logit rank of the Token-DiFR claim counted in the pass: everything else unchanged
    ar = difr.gumbel_score(logits, T, seeds, sid, pos, cg, V=V, temperatures=temps, want_rank=True)
    ra, rb = difr.score_both(logits, T, seeds, sid, pos, cg, ci, V=V, temperatures=temps, want_rank=True)
    torch.cuda.synchronize()
    assert "logit_rank" in ra
    _same_outputs(ra, {k: ar[k] for k in ra})
    _same_outputs(rb, {k: b[k] for k in rb})
    # the variant for concentrated rows (a test in front of the noise generation): the same, bit for bit
    pa, pb = difr.score_both_peaked(logits, T, seeds, sid, pos, cg, ci, V=V, temperatures=temps)
    torch.cuda.synchronize()
    _same_outputs(pa, {k: a[k] for k in pa})
    _same_outputs(pb, {k: b[k] for k in pb})
    # and with the sampler's own token and the Gaussian log-mass of the Token-IPT-DiFR side
    bt = difr.ipt_score(logits, T, seeds, sid, pos, ci, V=V, temperatures=temps, want_token=True, want_log_mass=True, sigma=0.05)
    ta, tb = difr.score_both(logits, T, seeds, sid, pos, cg, ci, V=V, temperatures=temps, want_token=True, want_log_mass=True,
                             sigma=0.05)
    torch.cuda.synchronize()
    assert "ipt_token" in tb and "log_mass" in tb
    _same_outputs(ta, {k: a[k] for k in ta})
    _same_outputs(tb, {k: bt[k] for k in tb})
    if case == "honest":
        assert (fa["flags"] & 1).all()
        assert int((fb["flags"] & 1).sum()) >= N - 2     # u within rounding of an interval end may fall either way


@pytest.mark.parametrize("dtype,V,ld,offset", [(torch.bfloat16, 20504, 20504, 0), (torch.bfloat16, 4099, 4099, 1),
                                               (torch.float32, 4100, 4104, 0), (torch.float32, 3001, 3001, 1)])
def test_logit_rank_and_classifier(difr, dtype, V, ld, offset):
    """Logit rank of the claimed token (an integer count: bit-exact) from both score kernels and from the
    unfiltered reference, and the three-class classifier with its exfiltratable-bits output."""
    N = 96
    g = torch.Generator(device=DEV).manual_seed(4321 + V)
    store = torch.randn(N * ld + offset + 8, generator=g, device=DEV, dtype=torch.float32).mul_(3.0).to(dtype)
    logits = store[offset:offset + N * ld].view(N, ld)
    logits[:, 5] = logits[:, 9]                                     # exact ties in every row
    logits[0, :40] = 0.0
    logits[0, 40:80] = -0.0                                         # signed zeros compare equal
    logits[1, 100:900] = float("-inf")
    wl = W.scaled(W.C1_TINY, S=3, L=32, V=V, chunk_rows=96)
    seeds, sid, pos, _ = _aux(wl)
    cpu_gen = torch.Generator().manual_seed(V)
    claims = torch.randint(0, V, (N,), generator=cpu_gen, dtype=torch.int32)
    claims[0], claims[1], claims[2], claims[3], claims[4], claims[5] = 3, 50, 5, 9, -1, V
    top = logits[:, :V].float().topk(4, dim=1).indices.cpu()
    claims[6:30] = top[6:30, 0].to(torch.int32)                     # highest logit: rank 0
    claims[30:50] = top[30:50, 3].to(torch.int32)                   # rank 3
    claims = claims.to(DEV)
    host = parity.to_host_logits(logits)
    want = oracle.logit_rank(host, V, claims.cpu().numpy())
    assert want[0] == int((logits[0, :V].float() > 0).sum()) and want[4] == -1 and want[5] == -1
    assert (want[6:30] == 0).all()
    a = difr.gumbel_score(logits, 0.9, seeds, sid, pos, claims, V=V, want_rank=True)
    b = difr.gumbel_score(logits, 0.9, seeds, sid, pos, claims, V=V, want_rank=True, unfiltered=True)
    c = difr.ipt_score(logits, 0.9, seeds, sid, pos, claims, V=V, want_rank=True)
    plain = difr.gumbel_score(logits, 0.9, seeds, sid, pos, claims, V=V)
    for out in (a, b, c):
        assert np.array_equal(out["logit_rank"].cpu().numpy(), want)
    _same_outputs({k: v for k, v in a.items() if k != "logit_rank"}, plain)      # asking for the rank changes nothing else
    # classifier on the library's own scores and ranks against the oracle on the oracle's
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    og = oracle.gumbel_score(host, V, f32(0.9), hs, hsid, hpos, claims.cpu().numpy())
    tau = np.float32(0.75)
    for R in (0, 1, 4, 8):
        got = difr.classify(a["margin"], a["logit_rank"], float(tau), R, V)
        ref = oracle.classify(og["margin"], want, tau, R, V)
        near = np.abs(np.nan_to_num(og["margin"], nan=np.inf) - tau) <= parity.TIE_REL * max(1.0, abs(float(tau)))
        diff = got["cls"].cpu().numpy() != ref["cls"]
        assert not (diff & ~near).any()
        assert np.allclose(got["bits"].cpu().numpy()[~diff], ref["bits"][~diff], atol=1e-6)
        if R == 8:
            cls = ref["cls"]
            assert (cls == 0).any() and (cls == 1).any() and (cls == 2).any()
    adm = torch.rand(N, generator=cpu_gen).to(DEV)
    got = difr.classify(a["margin"], a["logit_rank"], float(tau), 8, V, adm)
    ref = oracle.classify(og["margin"], want, tau, 8, V, adm.cpu().numpy().astype(np.float64))
    assert np.allclose(got["bits"].cpu().numpy(), ref["bits"], atol=1e-6)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("slope,shift", [(3.0, 0.0), (6.0, 30.0), (3.0, -50.0), (0.5, 0.0)])
def test_score_both_peaked_on_concentrated_rows(difr, dtype, slope, shift):
    """difr_score_both_peaked on the rows it is meant for (logits falling off as -slope ln rank: most wave-rounds are
    skipped before their noise is generated), shifted up and down (the test's cap on either side of zero), and on
    flat rows: bit-identical to difr_score_both, claims honest, random and absent."""
    N, V = 48, 20504
    g = torch.Generator().manual_seed(int(slope * 10) + int(shift) + 200)
    ranks = torch.argsort(torch.rand(N, V, generator=g), dim=1).float() + 1.0
    x = -slope * ranks.log() + torch.randn(N, V, generator=g) + shift
    E = 8 if dtype == torch.bfloat16 else 4
    logits = x.to(dtype).to(DEV)
    assert V % E == 0
    seeds = torch.tensor([77, -3], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    for T in (1.0, 0.3):
        honest = difr.gumbel_score(logits, T, seeds, sid, pos, None, want_scores=False)["argmax"]
        rnd = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
        for cg in (honest, rnd, None):
            a, b = difr.score_both(logits, T, seeds, sid, pos, cg, cg, want_token=True)
            pa, pb = difr.score_both_peaked(logits, T, seeds, sid, pos, cg, cg, want_token=True)
            torch.cuda.synchronize()
            _same_outputs(pa, a)
            _same_outputs(pb, b)
