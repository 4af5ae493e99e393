"""difr_score_both_filtered against the two calls it fuses (difr_gumbel_likelihood and difr_ipt_score_filtered, each
of which has its own parity tests against the oracle): every output must be identical, bit for bit, on shapes that
cover small and large selections, both storage types, ragged rows, sorted rows (the selection's worst case), invalid
claims, per-row temperatures and sampling mode."""
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def difr():
    import paper_2511_02620_amd as m
    m.load_library()
    return m


def _same(a, b, what):
    assert set(a) == set(b), (what, sorted(a), sorted(b))
    for k in a:
        x, y = a[k], b[k]
        assert torch.equal(torch.nan_to_num(x.float(), nan=-7.0), torch.nan_to_num(y.float(), nan=-7.0)), (what, k)


@pytest.mark.parametrize("dtype,V,k,p,s,order", [
    (torch.bfloat16, 20504, 50, 0.95, 16, "random"),      # the paper's policy: small buffers
    (torch.bfloat16, 20504, 50, 1.0, 0, "random"),        # empty active set
    (torch.bfloat16, 20504, 256, 0.5, 64, "random"),      # large selection: big buffers
    (torch.bfloat16, 20504, 50, 0.9, 16, "ascending"),    # every epoch runs full
    (torch.bfloat16, 2051, 7, 0.8, 5, "random"),          # ragged: one round and a tail
    (torch.bfloat16, 296, 50, 0.95, 16, "random"),        # fewer entries than one round
    (torch.float32, 5003, 20, 0.9, 8, "ties"),            # coarse logits: many equal keys
    (torch.float32, 9004, 64, 0.95, 64, "descending"),
    (torch.bfloat16, 20504, 0, 0.9, 16, "random"),        # the bare nucleus: its own search, then the estimator's pass
    (torch.float32, 5003, 0, 0.6, 8, "ties"),
])
def test_fused_pass_equals_the_two_calls(difr, dtype, V, k, p, s, order):
    N = 40
    g = torch.Generator().manual_seed(5 + V + k + s)
    x = torch.randn(N, V, generator=g) * 2.0
    if order == "ascending":
        x = x.sort(dim=1).values
    elif order == "descending":
        x = x.sort(dim=1, descending=True).values
    elif order == "ties":
        x = torch.round(x * 2) / 2
    ld = ((V + 7) // 8) * 8
    logits = torch.full((N, ld), float("nan"), dtype=dtype, device=DEV)
    logits[:, :V] = x.to(dtype).to(DEV)
    seeds = torch.tensor([21, 1 << 45, 3], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 3).to(torch.int32).to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    temps = torch.linspace(0.5, 1.3, N, device=DEV)
    z = torch.randn(96, generator=g).to(DEV)
    top = logits[:, :V].float().argmax(dim=1).to(torch.int32)
    cg = torch.where(torch.arange(N, device=DEV) % 2 == 0, top, torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV))
    ci = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    ci = torch.where(torch.arange(N, device=DEV) % 3 == 0, top, ci)
    cg[3] = V          # out of range
    ci[4] = -1
    for claims_ipt in (ci, None):   # scoring, and sampling mode on the IPT side
        lik, ipt = difr.score_both_filtered(logits, 1.0, seeds, sid, pos, cg, claims_ipt, z, top_k=k, top_p=p, s=s,
                                            sigma=0.4, temperatures=temps, V=V, want_active=s > 0, want_token=True,
                                            want_log_mass=True, sigma_ipt=0.02)
        lik1 = difr.gumbel_likelihood(logits, 1.0, seeds, sid, pos, cg, z, top_k=k, top_p=p, s=s, sigma=0.4,
                                      temperatures=temps, V=V, want_active=s > 0)
        ipt1 = difr.ipt_score_filtered(logits, 1.0, seeds, sid, pos, claims_ipt, top_k=k, top_p=p, temperatures=temps, V=V,
                                       want_token=True, want_log_mass=True, sigma=0.02)
        torch.cuda.synchronize()
        _same(lik, lik1, "likelihood side")
        _same(ipt, ipt1, "filtered IPT side")


def test_rejected_rows_and_bad_sequence_ids(difr):
    N, V = 16, 4096
    g = torch.Generator().manual_seed(9)
    logits = (torch.randn(N, V, generator=g) * 2).to(torch.bfloat16).to(DEV)
    logits[2, 100] = float("nan")
    logits[5, 7] = float("inf")
    seeds = torch.tensor([5, 6], dtype=torch.int64).to(DEV)
    sid = (torch.arange(N) % 2).to(torch.int32)
    sid[9] = 7              # no such sequence
    sid = sid.to(DEV)
    pos = torch.arange(N, dtype=torch.int32).to(DEV)
    temps = torch.full((N,), 0.8, device=DEV)
    temps[11] = 0.0         # unusable temperature
    z = torch.randn(32, generator=g).to(DEV)
    c = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    lik, ipt = difr.score_both_filtered(logits, 1.0, seeds, sid, pos, c, c, z, top_k=20, top_p=0.9, s=4, sigma=0.3,
                                        temperatures=temps, want_active=True, want_token=True, want_log_mass=True)
    lik1 = difr.gumbel_likelihood(logits, 1.0, seeds, sid, pos, c, z, top_k=20, top_p=0.9, s=4, sigma=0.3,
                                  temperatures=temps, want_active=True)
    ipt1 = difr.ipt_score_filtered(logits, 1.0, seeds, sid, pos, c, top_k=20, top_p=0.9, temperatures=temps,
                                   want_token=True, want_log_mass=True)
    torch.cuda.synchronize()
    _same(lik, lik1, "likelihood side")
    _same(ipt, ipt1, "filtered IPT side")
    assert (ipt["flags"][[2, 5, 9, 11]] != 0).all() and (lik["flags"][[2, 5, 9, 11]] != 0).all()
