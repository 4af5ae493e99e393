"""GPU parity of difr_admissible_count against the oracle.  The count is an integer decided by fp32
comparisons (max_score - y_v <= delta, the way the kernel forms margins); the oracle decides in double,
so the GPU's count must lie between the oracle's counts at delta -/+ 2e-5 (ten times the worst fp32
score error observed), and equal it whenever those two agree."""
import sys

import numpy as np
import pytest
import torch

import oracle
import parity
from paper_2511_02620_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-5


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def difr():
    import paper_2511_02620_amd as m
    m.load_library()
    return m


def _check(difr, logits, V, T, seeds, sid, pos, delta, temps=None):
    g = difr.gumbel_score(logits, T, seeds, sid, pos, None, V=V, temperatures=temps)
    a = difr.admissible_count(logits, T, seeds, sid, pos, g["max_score"], delta, V=V, temperatures=temps)
    torch.cuda.synchronize()
    host = parity.to_host_logits(logits)
    o = oracle.admissible_count(host, V, np.float32(T), parity.seeds_u64(seeds), sid.cpu().numpy(),
                                parity.positions_u32(pos), delta, tol=TOL,
                                temperatures=None if temps is None else temps.cpu().numpy())
    c = a["count"].cpu().numpy()
    assert (c >= o["count_lo"]).all() and (c <= o["count_hi"]).all(), np.nonzero((c < o["count_lo"]) | (c > o["count_hi"]))[0][:10]
    sure = o["count_lo"] == o["count_hi"]
    assert (c[sure] == o["count"][sure]).all()
    l2 = a["log2_count"].cpu().numpy()
    assert np.allclose(l2, np.log2(c.astype(np.float64)), atol=1e-5)
    return c, int((~sure).sum())


@pytest.mark.parametrize("dtype,V,ld,offset,delta", [
    (torch.bfloat16, 20504, 20504, 0, 3.0),      # 10 full rounds + a partial one
    (torch.bfloat16, 20504, 20504, 0, 0.0),
    (torch.bfloat16, 16384, 16384, 0, 6.0),
    (torch.bfloat16, 2051, 2056, 0, 2.0),        # ragged last vector
    (torch.float32, 5003, 5004, 0, 4.0),
    (torch.bfloat16, 4099, 4099, 1, 2.5),        # unaligned rows: every entry evaluated
    (torch.bfloat16, 300, 304, 0, 50.0),         # delta beyond every margin: the whole vocabulary
])
def test_admissible_count_every_row(difr, dtype, V, ld, offset, delta):
    N = 64
    g = torch.Generator().manual_seed(321 + V)
    store = torch.empty(N * ld + offset + 8, dtype=dtype, device=DEV)
    logits = store[offset:offset + N * ld].view(N, ld)
    logits[:, :V] = (torch.randn(N, V, generator=g) * 2.0).to(dtype).to(DEV)
    seeds = torch.tensor([0x1234ABCD00000077, 5], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    c, unsure = _check(difr, logits, V, 0.8, seeds, sid, pos, delta)
    say("admissible", dtype, V, delta, "mean count %.2f, max %d, near-threshold rows %d" % (c.mean(), c.max(), unsure))
    assert (c >= 1).all()
    if delta == 0.0:
        assert (c == 1).all()
    if delta == 50.0:
        assert (c == V).all()


def test_admissible_count_c2_class_rows_and_claimed_consistency(difr):
    """Zipf-profile rows at V = 128256 with per-row temperatures; the claimed token's own margin decides
    whether it is inside the set the count describes."""
    wl = W.scaled(W.C2_3B, S=2, L=48, chunk_rows=96)
    ver, prov = wl.logits_chunk(0, DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    temps = torch.linspace(0.5, 1.5, wl.N).to(DEV)
    delta = 2.0
    c, unsure = _check(difr, ver, wl.V, wl.temperature, seeds, sid, pos, delta, temps=temps)
    say("admissible C2-class: mean count %.2f, near-threshold rows %d" % (c.mean(), unsure))
    # masking a claimed token removes exactly one admissible token iff its margin was <= delta
    gen = torch.Generator().manual_seed(9)
    claims = torch.randint(0, wl.V, (wl.N,), generator=gen, dtype=torch.int32).to(DEV)
    top = ver.float().topk(3, dim=1).indices[:, 2].to(torch.int32)
    claims = torch.where(torch.arange(wl.N, device=DEV) % 2 == 0, top, claims)
    g = difr.gumbel_score(ver, wl.temperature, seeds, sid, pos, claims, temperatures=temps)
    masked = ver.clone()
    masked[torch.arange(wl.N, device=DEV), claims.long()] = float("-inf")
    a0 = difr.admissible_count(ver, wl.temperature, seeds, sid, pos, g["max_score"], delta, temperatures=temps)["count"]
    a1 = difr.admissible_count(masked, wl.temperature, seeds, sid, pos, g["max_score"], delta, temperatures=temps)["count"]
    torch.cuda.synchronize()
    assert torch.equal(a0 - a1, (g["margin"] <= delta).to(torch.int32))


def test_admissible_count_rejected_rows(difr):
    N, V = 8, 1024
    logits = torch.randn(N, V, device=DEV).to(torch.bfloat16)
    seeds = torch.tensor([1], dtype=torch.int64).to(DEV)
    sid = torch.zeros(N, dtype=torch.int32, device=DEV)
    sid[2] = 5                                                   # sequence id out of range
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    temps = torch.ones(N, device=DEV)
    temps[4] = -1.0                                              # unusable temperature
    g = difr.gumbel_score(logits, 1.0, seeds, sid, pos, None, temperatures=temps)
    a = difr.admissible_count(logits, 1.0, seeds, sid, pos, g["max_score"], 1.0, temperatures=temps)
    torch.cuda.synchronize()
    c = a["count"].cpu().numpy()
    assert c[2] == 0 and c[4] == 0 and (np.delete(c, [2, 4]) >= 1).all()
    assert torch.isnan(a["log2_count"][2]) and torch.isnan(a["log2_count"][4])


# ---- the one-pass variant: difr_score_both_admissible ----

def _one_pass(difr, logits, V, T, seeds, sid, pos, cg, ci, delta, temps=None):
    """Scores must be those of difr_score_both bit for bit; every determined count must be the two-pass count
    (same expression, same maximum) and lie inside the oracle's bracket.  Returns (counts, undetermined rows)."""
    g1, i1, a = difr.score_both_admissible(logits, T, seeds, sid, pos, delta, cg, ci, V=V, temperatures=temps)
    g0, i0 = difr.score_both(logits, T, seeds, sid, pos, cg, ci, V=V, temperatures=temps)
    two = difr.admissible_count(logits, T, seeds, sid, pos, g0["max_score"], delta, V=V, temperatures=temps)
    torch.cuda.synchronize()
    for d0, d1 in ((g0, g1), (i0, i1)):
        for k in d0:
            assert torch.equal(torch.nan_to_num(d0[k].float(), nan=-7.0), torch.nan_to_num(d1[k].float(), nan=-7.0)), k
    c = a["count"].cpu().numpy()
    det = c >= 0
    assert (c[det] == two["count"].cpu().numpy()[det]).all()
    host = parity.to_host_logits(logits)
    o = oracle.admissible_count(host, V, np.float32(T), parity.seeds_u64(seeds), sid.cpu().numpy(),
                                parity.positions_u32(pos), delta, tol=TOL,
                                temperatures=None if temps is None else temps.cpu().numpy())
    assert (c[det] >= o["count_lo"][det]).all() and (c[det] <= o["count_hi"][det]).all()
    l2 = a["log2_count"].cpu().numpy()
    assert np.allclose(l2[det], np.log2(c[det].astype(np.float64)), atol=1e-5) and np.isnan(l2[~det]).all()
    return c, int((~det).sum())


@pytest.mark.parametrize("dtype,V,ld,delta,claims", [
    (torch.bfloat16, 20504, 20504, 3.0, "honest"),
    (torch.bfloat16, 20504, 20504, 0.0, "honest"),
    (torch.bfloat16, 20504, 20504, 5.0, "random"),     # the bound starts far below the maximum
    (torch.bfloat16, 20504, 20504, 2.5, "none"),       # sampling mode: the bound starts at -inf
    (torch.bfloat16, 2051, 2056, 2.0, "random"),       # ragged last vector
    (torch.float32, 5003, 5004, 4.0, "honest"),
    (torch.float32, 5003, 5004, 1.0, "none"),
    (torch.bfloat16, 300, 304, 1.5, "random"),         # a single, partly filled round
])
def test_one_pass_count_every_row(difr, dtype, V, ld, delta, claims):
    N = 96
    g = torch.Generator().manual_seed(77 + V + len(claims))
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)
    logits[:, :V] = (torch.randn(N, V, generator=g) * 2.0).to(dtype).to(DEV)
    seeds = torch.tensor([0x1234ABCD00000077, 5, 1 << 40], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 3).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    if claims == "honest":
        cg = difr.gumbel_score(logits, 0.8, seeds, sid, pos, None, V=V, want_scores=False)["argmax"]
    elif claims == "random":
        cg = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    else:
        cg = None
    ci = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    c, undet = _one_pass(difr, logits, V, 0.8, seeds, sid, pos, cg, ci, delta)
    say("one-pass admissible", dtype, V, delta, claims, "mean count %.2f, undetermined rows %d of %d" % (c[c >= 0].mean(), undet, N))
    assert undet == 0


def test_one_pass_count_reports_what_it_cannot_hold(difr):
    """A delta wider than every margin makes every token a candidate: more than the on-chip lists hold.  The rows
    must come back as undetermined (-1), never as a wrong count; a vocabulary that fits is counted whole."""
    N, V = 32, 20504
    g = torch.Generator().manual_seed(9)
    logits = (torch.randn(N, V, generator=g) * 2.0).to(torch.bfloat16).to(DEV)
    seeds = torch.tensor([3], dtype=torch.int64).to(DEV)
    sid = torch.zeros(N, dtype=torch.int32, device=DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    c, undet = _one_pass(difr, logits, V, 1.0, seeds, sid, pos, None, None, 60.0)
    assert undet == N
    small = logits[:, :1000].contiguous()
    c, undet = _one_pass(difr, small, 1000, 1.0, seeds, sid, pos, None, None, 60.0)
    assert undet == 0 and (c == 1000).all()


def test_one_pass_count_c2_class_rows(difr):
    """Zipf-profile rows at V = 128256, honest claims with a few swapped tokens, per-row temperatures."""
    wl = W.scaled(W.C2_3B, S=2, L=64, chunk_rows=128)
    ver, prov = wl.logits_chunk(0, DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    temps = torch.linspace(0.5, 1.3, wl.N, device=DEV)
    cg = difr.gumbel_score(prov, 1.0, seeds, sid, pos, None, temperatures=temps, want_scores=False)["argmax"]
    cg[::9] = (cg[::9] + 12345) % wl.V
    ci = difr.ipt_score(prov, 1.0, seeds, sid, pos, None, temperatures=temps, want_token=True, want_interval=False)["ipt_token"]
    for delta in (1.0, 2.5, 5.0):
        c, undet = _one_pass(difr, ver, wl.V, 1.0, seeds, sid, pos, cg, ci, delta, temps=temps)
        say("one-pass admissible C2 rows, delta", delta, "mean count %.2f max %d undetermined %d" % (c[c >= 0].mean(), c.max(), undet))
        assert undet == 0
