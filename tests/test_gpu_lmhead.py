"""GPU parity of the fused LM-head path (difr_lmhead_score) against the oracle's double-precision
product followed by the two estimators, on every row of small cases that span several token blocks,
several vocabulary tiles and ranges, and ragged ends in both directions."""
import dataclasses
import sys

import numpy as np
import pytest
import torch

import oracle
import parity
from paper_2511_02620_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# The logits are fp32 matrix-core sums of d bf16 products: their error against the oracle's double sum
# is a few ulp of the partial sums (|x| up to ~10 here, so ~1e-5).  Decisions closer than that to a
# tie may fall either way; they are excused and counted.
TIE = 3e-5


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def difr():
    import paper_2511_02620_amd as m
    m.load_library()
    return m


def bits(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _case(S, L, V, d, T=1.0, w_sigma=None):
    return dataclasses.replace(W.C4_LMHEAD, S=S, L=L, V=V, d=d, temperature=T,
                               w_sigma=(2.0 / d ** 0.5) if w_sigma is None else w_sigma)


@pytest.mark.parametrize("S,L,V,d,mode", [
    (2, 150, 1000, 128, "mutated"),       # 2 token blocks (second ragged), 4 tiles (last ragged), 4 ranges
    (1, 256, 2088, 256, "honest"),        # exactly one token block, 9 tiles
    (3, 200, 5000, 192, "mutated"),       # 3 token blocks, 20 tiles
    (1, 40, 300, 64, "sampling"),         # less than one tile either way, no claims
    (2, 130, 1500, 128, "per_row_T"),
    (1, 100, 777, 64, "invalid"),
])
def test_lmhead_every_row(difr, S, L, V, d, mode):
    wl = _case(S, L, V, d, T=0.8)
    Wm = wl.weight(DEV)
    Hv, Hp = wl.hidden(DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    N = wl.N
    temps = torch.linspace(0.5, 1.7, N).to(DEV) if mode == "per_row_T" else None
    say("lmhead case", S, L, V, d, mode)
    # honest claims: the library's own samplers on the prover's hidden states
    g0, i0 = difr.lmhead_score(Hp, Wm, wl.temperature, seeds, sid, pos, None, None, temperatures=temps)
    cg = g0["argmax"].clone()
    # the IPT sampler's token from the oracle (the fused path has no honest-token output)
    hs, hsid, hpos = parity.seeds_u64(seeds), sid.cpu().numpy(), parity.positions_u32(pos)
    htemps = None if temps is None else temps.cpu().numpy()
    _, oi0 = oracle.lmhead_score(bits(Hp), bits(Wm), np.float32(wl.temperature), hs, hsid, hpos, None, None,
                                 temperatures=htemps)
    ci = torch.from_numpy(oi0["ipt_token"]).to(DEV)
    gen = torch.Generator().manual_seed(5 + V)
    if mode in ("mutated", "per_row_T"):
        k = torch.arange(N, device=DEV)
        cg = torch.where(k % 4 == 1, torch.randint(0, V, (N,), generator=gen, dtype=torch.int32).to(DEV), cg)
        ci = torch.where(k % 4 == 2, torch.randint(0, V, (N,), generator=gen, dtype=torch.int32).to(DEV), ci)
    elif mode == "invalid":
        cg = cg.clone(); ci = ci.clone()
        cg[::3] = -1; ci[1::3] = V; cg[2::3] = V + 7
    elif mode == "sampling":
        cg = ci = None
    g, i = difr.lmhead_score(Hv, Wm, wl.temperature, seeds, sid, pos, cg, ci, temperatures=temps)
    torch.cuda.synchronize()
    og, oi = oracle.lmhead_score(bits(Hv), bits(Wm), np.float32(wl.temperature), hs, hsid, hpos,
                                 None if cg is None else cg.cpu().numpy(), None if ci is None else ci.cpu().numpy(),
                                 temperatures=htemps)
    sg = parity.compare_gumbel(g, og, tie_rel=TIE)
    si = parity.compare_ipt(i, oi, tie_rel=TIE)
    say("  gumbel", sg, "ipt", si)
    if mode == "honest":
        # the verifier's hidden states differ from the prover's by drift only: most claims still match
        assert float((g["flags"] & 1).float().mean()) > 0.9
    # same call again: bit-identical
    g2, i2 = difr.lmhead_score(Hv, Wm, wl.temperature, seeds, sid, pos, cg, ci, temperatures=temps)
    torch.cuda.synchronize()
    for a, b in ((g, g2), (i, i2)):
        for key in a:
            assert torch.equal(torch.nan_to_num(a[key].float(), nan=-7.0), torch.nan_to_num(b[key].float(), nan=-7.0)), key


def test_lmhead_honest_claim_on_identical_inputs_has_margin_zero(difr):
    """A claim sampled by the same kernel from the same hidden states is the row maximum again:
    margin exactly 0 and MATCH, whatever the accumulation order of the matrix cores is."""
    wl = _case(2, 160, 3000, 128, T=1.0)
    Wm = wl.weight(DEV)
    Hv, _ = wl.hidden(DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    g0, _ = difr.lmhead_score(Hv, Wm, wl.temperature, seeds, sid, pos, None, None)
    g, _ = difr.lmhead_score(Hv, Wm, wl.temperature, seeds, sid, pos, g0["argmax"], None)
    torch.cuda.synchronize()
    assert torch.equal(g["argmax"], g0["argmax"])
    assert (g["margin"] == 0).all() and (g["flags"] & 1).all()
    assert torch.equal(g["max_score"], g["claimed_score"])


def test_lmhead_agrees_with_stored_logit_path_on_exact_products(difr):
    """Small-integer inputs make every product and partial sum exact in fp32, so the logits equal the
    integer matrix product in any accumulation order, and the fused path must reproduce
    difr_score_both on those logits stored as fp32: scores to the last bit."""
    gen = torch.Generator().manual_seed(99)
    N, V, d = 300, 1300, 128
    Hi = torch.randint(-4, 5, (N, d), generator=gen)
    Wi = torch.randint(-8, 9, (V, d), generator=gen)
    H = Hi.to(torch.bfloat16).to(DEV)
    Wm = (Wi.float() / 32.0).to(torch.bfloat16).to(DEV)
    logits = ((Hi @ Wi.T).float() / 32.0).to(DEV)          # |sum| <= 128*4*8 = 4096: exact
    seeds = torch.tensor([11, -5, 1 << 40], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 3).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    T = 0.9
    cg = torch.randint(0, V, (N,), generator=gen, dtype=torch.int32).to(DEV)
    ci = torch.randint(0, V, (N,), generator=gen, dtype=torch.int32).to(DEV)
    g, i = difr.lmhead_score(H, Wm, T, seeds, sid, pos, cg, ci)
    gs, is_ = difr.score_both(logits, T, seeds, sid, pos, cg, ci)
    torch.cuda.synchronize()
    for key in ("margin", "argmax", "max_score", "claimed_score", "flags"):
        assert torch.equal(g[key], gs[key]), key
    assert torch.equal(i["u"], is_["u"]) and torch.equal(i["flags"], is_["flags"])
    # the softmax sums are accumulated in a different order: equal to fp32 rounding, not to the bit
    for key in ("dist", "cdf_lo", "cdf_hi"):
        assert float((i[key] - is_[key]).abs().max()) <= 2e-6, key
