"""GPU parity of difr_ipt_score_filtered against the oracle: kept-set size bit-exact, interval ends and
distance within 1e-4 (observed ~1e-8: the kernel works in fp64 on at most 256 tokens), MATCH and the sampler's
token equal except where u lies within 1e-6 of an interval end (excused and counted)."""
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


def _compare(difr, logits, V, T, seeds, sid, pos, claims, k, p, temps=None):
    out = difr.ipt_score_filtered(logits, T, seeds, sid, pos, claims, top_k=k, top_p=p, temperatures=temps, V=V,
                                  want_token=True, want_log_mass=True, sigma=0.02)
    torch.cuda.synchronize()
    host = parity.to_host_logits(logits)
    ref = oracle.ipt_filtered_score(host, V, np.float32(T), parity.seeds_u64(seeds), sid.cpu().numpy(),
                                    parity.positions_u32(pos), None if claims is None else claims.cpu().numpy(), k,
                                    float(np.float32(p)), temperatures=None if temps is None else temps.cpu().numpy(),
                                    sigma=0.02)
    assert np.array_equal(out["kept"].cpu().numpy(), ref["kept"]), "kept-set size differs"
    st = parity.compare_ipt({k2: v for k2, v in out.items() if k2 not in ("kept", "ipt_token")}, ref, log_mass_sigma=0.02)
    tok, rt = out["ipt_token"].cpu().numpy(), ref["ipt_token"]
    diff = tok != rt
    # the sampler's token may differ only when u sits on a CDF step: check with the oracle that the GPU's token's
    # own interval touches u
    excused = 0
    for r in np.nonzero(diff)[0]:
        one = oracle.ipt_filtered_score(host[r:r + 1], V, np.float32(T) if temps is None else float(temps[r]),
                                        parity.seeds_u64(seeds), sid.cpu().numpy()[r:r + 1], parity.positions_u32(pos)[r:r + 1],
                                        np.array([tok[r]], np.int32), k, float(np.float32(p)))
        assert one["dist"][0] < 1e-6 and one["cdf_hi"][0] > one["cdf_lo"][0], (r, tok[r], rt[r])
        excused += 1
    st["token_excused"] = excused
    st["mean_kept"] = float(ref["kept"].mean())
    return st, out


@pytest.mark.parametrize("dtype,V,k,p,order", [
    (torch.bfloat16, 20504, 50, 0.95, "random"),
    (torch.bfloat16, 20504, 50, 1.0, "random"),
    (torch.bfloat16, 20504, 256, 0.5, "ascending"),
    (torch.bfloat16, 20504, 50, 0.9, "ascending"),   # small buffers: every epoch runs full and is repeated wave by wave
    (torch.float32, 9004, 64, 0.95, "ascending"),
    (torch.bfloat16, 16384, 1, 1.0, "random"),
    (torch.bfloat16, 2056, 7, 0.8, "descending"),
    (torch.bfloat16, 296, 50, 0.95, "random"),
    (torch.float32, 5004, 20, 0.9, "ties"),
])
def test_ipt_filtered_every_row(difr, dtype, V, k, p, order):
    N = 64
    g = torch.Generator().manual_seed(11 + V + k)
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
    honest = difr.ipt_score_filtered(logits, T, seeds, sid, pos, None, top_k=k, top_p=p, want_token=True)["ipt_token"]
    claims = honest.clone()
    i = torch.arange(N, device=DEV)
    claims = torch.where(i % 4 == 1, torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV), claims)
    claims = torch.where(i % 4 == 2, logits.float().topk(min(3, V), dim=1).indices[:, -1].to(torch.int32), claims)
    claims[5] = -1
    claims[9] = V
    st, out = _compare(difr, logits, V, T, seeds, sid, pos, claims, k, p)
    say("ipt filtered", dtype, V, "k=%d p=%g %s:" % (k, p, order), st)
    honest_rows = (i % 4 == 0) | (i % 4 == 3)
    honest_rows[5] = honest_rows[9] = False
    assert (out["flags"][honest_rows] & 1).all() and (out["dist"][honest_rows] == 0).all()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("k,p", [(150, 1.0), (256, 0.8), (101, 1.0)])
def test_ipt_filtered_signed_zeros_tie_by_index(difr, dtype, k, p):
    """-0 and +0 are the same logit: a top-k (or top-p) cut that falls among zeros of both signs takes them in index
    order whatever their sign."""
    N, V = 32, 4000
    g = torch.Generator().manual_seed(19)
    x = torch.full((N, V), -3.0)
    for r in range(N):
        perm = torch.randperm(V, generator=g)
        x[r, perm[:100]] = 2.0
        x[r, perm[100:2100]] = torch.where(torch.rand(2000, generator=g) < 0.5, torch.tensor(0.0), torch.tensor(-0.0))
    logits = x.to(dtype).to(DEV)
    seeds = torch.tensor([23], dtype=torch.int64).to(DEV)
    sid = torch.zeros(N, dtype=torch.int32, device=DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    honest = difr.ipt_score_filtered(logits, 1.0, seeds, sid, pos, None, top_k=k, top_p=p, want_token=True)["ipt_token"]
    rnd = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    claims = torch.where(torch.arange(N, device=DEV) % 2 == 0, honest, rnd)
    st, out = _compare(difr, logits, V, 1.0, seeds, sid, pos, claims, k, p)
    say("filtered signed zeros", dtype, k, p, st)
    assert st["token_excused"] == 0


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("V,k", [(107, 50), (107, 65), (3003, 50), (3003, 200), (9007, 256)])
def test_ipt_filtered_masked_rows_with_a_ragged_end(difr, dtype, V, k):
    """Rows in which most entries are masked (-inf), so that the k-th largest logit so far is a masked entry for much of
    the pass (the selection's threshold is then the image of -inf), with finite entries in the ragged last vector:
    every finite entry must still reach the selection (top_p just below 1 makes the kept count feel each of them)."""
    N = 48
    g = torch.Generator().manual_seed(5 + V + k)
    x = torch.randn(N, V, generator=g) * 2.0
    x[torch.rand(N, V, generator=g) < 0.6] = float("-inf")
    x[:, V - 3:] = torch.randn(N, 3, generator=g) + 1.0       # finite, and not small, in the last vector
    E = 8 if dtype == torch.bfloat16 else 4
    ld = ((V + E - 1) // E) * E
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)
    logits[:, :V] = x.to(dtype).to(DEV)
    seeds = torch.tensor([77, -9], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    temps = torch.linspace(0.5, 1.4, N).to(DEV)
    for p in (0.999, 0.9):
        st, out = _compare(difr, logits, V, 1.3, seeds, sid, pos, None, k, p, temps=temps)
        say("filtered masked ragged", dtype, V, k, p, st)


def test_ipt_filtered_c2_class_rows(difr):
    wl = W.scaled(W.C2_3B, S=2, L=32, chunk_rows=64)
    ver, prov = wl.logits_chunk(0, DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    temps = torch.linspace(0.6, 1.2, wl.N).to(DEV)
    claims = difr.ipt_score_filtered(prov, wl.temperature, seeds, sid, pos, None, top_k=50, top_p=0.95, temperatures=temps,
                                     want_token=True)["ipt_token"]
    st, out = _compare(difr, ver, wl.V, wl.temperature, seeds, sid, pos, claims, 50, 0.95, temps=temps)
    say("ipt filtered C2-class:", st, "match rate %.3f" % float((out["flags"] & 1).float().mean()))
