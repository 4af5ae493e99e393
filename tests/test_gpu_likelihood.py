"""GPU parity of difr_gumbel_likelihood against the oracle: the active set S and the filter threshold tau
must be the oracle's (S is chosen on fp32 scores: a row whose oracle gap between the last member of S and the
first token left out is below 1e-5 may differ and is excused and counted), pi within 1e-4 absolute and
ln pi within 1e-3 where pi > 1e-30."""
import sys

import numpy as np
import pytest
import torch

import oracle
import parity
from paper_2511_02620_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def difr():
    import paper_2511_02620_amd as m
    m.load_library()
    return m


def _compare(difr, logits, V, T, seeds, sid, pos, claims, k, p, s, sigma, M=384, temps=None):
    z = torch.randn(M, generator=torch.Generator().manual_seed(1000 + s + k), dtype=torch.float32)
    out = difr.gumbel_likelihood(logits, T, seeds, sid, pos, claims, z.to(DEV), top_k=k, top_p=p, s=s, sigma=sigma,
                                 temperatures=temps, V=V, want_active=s > 0)
    out2 = difr.gumbel_likelihood(logits, T, seeds, sid, pos, claims, z.to(DEV), top_k=k, top_p=p, s=s, sigma=sigma,
                                  temperatures=temps, V=V, want_active=s > 0)
    torch.cuda.synchronize()
    for key in out:                                                  # run to run: bit-identical
        assert torch.equal(torch.nan_to_num(out[key].float(), nan=-7.0), torch.nan_to_num(out2[key].float(), nan=-7.0)), key
    ref = oracle.likelihood(parity.to_host_logits(logits), V, np.float32(T), parity.seeds_u64(seeds), sid.cpu().numpy(),
                            parity.positions_u32(pos), None if claims is None else claims.cpu().numpy(), k, float(np.float32(p)),
                            s, float(np.float32(sigma)), z.double().numpy(),
                            temperatures=None if temps is None else temps.cpu().numpy())
    pi, lp, tau = out["pi"].cpu().numpy().astype(np.float64), out["log_pi"].cpu().numpy().astype(np.float64), out["tau"].cpu().numpy()
    assert np.array_equal(tau, ref["tau"].astype(np.float32)), "filter threshold differs"
    excused = np.zeros(len(pi), bool)
    if s > 0:
        # S as a set: its members are listed by score, and two scores that differ by less than fp32 resolves (1e-6 at
        # a score of 60) are listed by index on the GPU and by value in the oracle; the estimate does not depend on it
        act = np.sort(out["active"].cpu().numpy(), axis=1)
        diff = (act != np.sort(ref["active"], axis=1)).any(axis=1)
        excused = diff & (ref["gap_s"] < 1e-5)
        assert not (diff & ~excused).any(), "active set differs on rows %s" % np.nonzero(diff & ~excused)[0][:10]
    both_nan = np.isnan(pi) & np.isnan(ref["pi"])
    err = np.where(both_nan | excused, 0.0, np.abs(pi - ref["pi"]))
    assert (err <= 1e-4).all(), "pi: worst %g at row %d (gpu %g oracle %g)" % (err.max(), err.argmax(), pi[err.argmax()], ref["pi"][err.argmax()])
    ok = (ref["pi"] > 1e-30) & ~excused
    lerr = np.abs(lp[ok] - ref["log_pi"][ok])
    assert (lerr <= 1e-3).all(), "ln pi: worst %g" % lerr.max()
    zero = (ref["pi"] == 0) & ~excused
    assert (pi[zero] == 0).all() and np.isneginf(lp[zero]).all()
    fl = out["flags"].cpu().numpy()
    want_invalid = np.isnan(ref["pi"])
    assert np.array_equal((fl & 2) != 0, want_invalid)
    return dict(rows=len(pi), excused=int(excused.sum()), pi_err=float(err.max()), lnpi_err=float(lerr.max()) if lerr.size else 0.0,
                mean_pi=float(np.nanmean(ref["pi"])))


@pytest.mark.parametrize("dtype,V,k,p,s,sigma,order", [
    (torch.bfloat16, 20504, 50, 0.95, 16, 0.5, "random"),
    (torch.bfloat16, 20504, 0, 1.0, 8, 1.0, "random"),
    (torch.bfloat16, 20504, 10, 1.0, 1, 0.2, "random"),
    (torch.bfloat16, 16384, 256, 0.5, 64, 0.05, "random"),
    (torch.bfloat16, 20504, 50, 0.9, 0, 0.5, "random"),
    (torch.bfloat16, 20504, 50, 0.95, 256, 0.5, "ascending"),      # every entry is a new maximum: worst case for the selection
    (torch.bfloat16, 20504, 50, 0.95, 16, 0.5, "ascending"),       # the same with the small buffers: epochs repeated wave by wave
    (torch.float32, 9004, 64, 0.9, 64, 0.5, "ascending"),
    (torch.bfloat16, 20504, 50, 0.95, 16, 0.5, "descending"),
    (torch.bfloat16, 2056, 7, 0.8, 5, 0.01, "random"),             # one round and a tail
    (torch.bfloat16, 296, 50, 0.95, 16, 0.5, "random"),            # fewer entries than one round
    (torch.float32, 5004, 50, 0.95, 16, 0.5, "random"),
    (torch.float32, 5004, 3, 0.5, 300 - 44, 2.0, "ties"),          # coarse logits: many equal keys
])
def test_likelihood_every_row(difr, dtype, V, k, p, s, sigma, order):
    N = 48
    g = torch.Generator().manual_seed(77 + V + s)
    x = torch.randn(N, V, generator=g) * 2.0
    if order == "ascending":
        x = x.sort(dim=1).values
    elif order == "descending":
        x = x.sort(dim=1, descending=True).values
    elif order == "ties":
        x = (x * 2).round() / 2
    logits = x.to(dtype).to(DEV)
    seeds = torch.tensor([0x1234ABCD00000077, -5], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    T = 0.9
    honest = difr.gumbel_score(logits, T, seeds, sid, pos, None)["argmax"]
    claims = honest.clone()
    rnd = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    top3 = logits.float().topk(3, dim=1).indices[:, 2].to(torch.int32)
    i = torch.arange(N, device=DEV)
    claims = torch.where(i % 4 == 1, rnd, claims)
    claims = torch.where(i % 4 == 2, top3, claims)
    claims[5] = -1
    claims[9] = V
    st = _compare(difr, logits, V, T, seeds, sid, pos, claims, k, p, s, sigma)
    say("likelihood", dtype, V, "k=%d p=%g s=%d sigma=%g %s:" % (k, p, s, sigma, order), st)


def test_likelihood_c2_class_rows(difr):
    """Zipf-profile rows at V = 128256 with the paper's generation policy (top-k 50, top-p 0.95) and per-row T."""
    wl = W.scaled(W.C2_3B, S=2, L=32, chunk_rows=64)
    ver, prov = wl.logits_chunk(0, DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    temps = torch.linspace(0.6, 1.2, wl.N).to(DEV)
    claims = difr.gumbel_score(prov, wl.temperature, seeds, sid, pos, None, temperatures=temps)["argmax"]
    claims = wl.mutate_claims(0, claims, ver)
    for sigma in (0.01, 0.3):
        st = _compare(difr, ver, wl.V, wl.temperature, seeds, sid, pos, claims, 50, 0.95, 16, sigma, temps=temps)
        say("likelihood C2-class sigma=%g:" % sigma, st)
