"""The whole hot path recorded into a HIP graph and replayed: the library allocates nothing, clears nothing
with memset nodes and never synchronises, so a caller may capture its calls.  Every replay (with the
program's own eager work and synchronisations in between, and new input contents each time) must give
exactly what the eager calls give on the same inputs."""
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
    for k in a:
        x, y = a[k], b[k]
        assert torch.equal(torch.nan_to_num(x.float(), nan=-7.0), torch.nan_to_num(y.float(), nan=-7.0)), (what, k)


def _inputs(seed, N, V, S):
    g = torch.Generator().manual_seed(seed)
    logits = (torch.randn(N, V, generator=g) * 2.5).to(torch.bfloat16)
    cg = torch.randint(0, V, (N,), generator=g, dtype=torch.int32)
    ci = torch.randint(0, V, (N,), generator=g, dtype=torch.int32)
    return logits, cg, ci


def test_row_path_replays_match_eager(difr):
    S, L, V = 6, 80, 8200          # ragged tail (V % 8 != 0), several rounds per row
    N = S * L
    seeds = torch.arange(1, S + 1, dtype=torch.int64).mul_(0x9E3779B97F4A7C15 % (1 << 62)).to(DEV)
    sid = torch.arange(N, dtype=torch.int32).div(L, rounding_mode="floor").to(torch.int32).to(DEV)
    pos = (torch.arange(N) % L).to(torch.int32).to(DEV)
    off = (torch.arange(S + 1, dtype=torch.int64) * L).to(DEV)
    logits = torch.empty(N, V, dtype=torch.bfloat16, device=DEV)
    cg = torch.empty(N, dtype=torch.int32, device=DEV)
    ci = torch.empty(N, dtype=torch.int32, device=DEV)
    zdraws = torch.randn(64, generator=torch.Generator().manual_seed(4)).to(DEV)

    def step():
        g, i = difr.score_both(logits, 0.8, seeds, sid, pos, cg, ci)
        pg = difr.seq_reduce(g["margin"], g["flags"], off, 0.05)
        pi = difr.seq_reduce(i["dist"], i["flags"], off, 0.01)
        a = difr.admissible_count(logits, 0.8, seeds, sid, pos, g["max_score"], 2.0)
        f = difr.ipt_score_filtered(logits, 0.8, seeds, sid, pos, ci, top_k=20, top_p=0.9)
        lk, fi = difr.score_both_filtered(logits, 0.8, seeds, sid, pos, cg, ci, zdraws, top_k=20, top_p=0.9, s=8, sigma=0.3)
        return g, i, pg, pi, a, f, lk, fi

    def load(seed):
        x, a, b = _inputs(seed, N, V, S)
        logits.copy_(x.to(DEV))
        cg.copy_(a.to(DEV))
        ci.copy_(b.to(DEV))

    load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):      # warm-up on the side stream, as graph capture wants
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = step()
    for rep, seed in enumerate((11, 12, 13, 14)):
        load(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [{k: v.clone() for k, v in d.items()} for d in captured]
        eager = step()                 # the program's own eager work between replays
        torch.cuda.synchronize()
        for d_got, d_eager, name in zip(got, eager, ("gumbel", "ipt", "pool_g", "pool_i", "admissible", "filtered", "likelihood", "filtered_fused")):
            _same(d_got, d_eager, "replay %d %s" % (rep, name))


def test_lmhead_replays_match_eager(difr):
    S, L, V, d = 3, 100, 1000, 128     # ragged token block and ragged vocabulary tile
    N = S * L
    g = torch.Generator().manual_seed(5)
    W = (torch.randn(V, d, generator=g) * 0.08).to(torch.bfloat16).to(DEV)
    H = torch.empty(N, d, dtype=torch.bfloat16, device=DEV)
    seeds = torch.tensor([7, 8, 9], dtype=torch.int64).to(DEV)
    sid = torch.arange(N, dtype=torch.int32).div(L, rounding_mode="floor").to(torch.int32).to(DEV)
    pos = (torch.arange(N) % L).to(torch.int32).to(DEV)
    cg = torch.empty(N, dtype=torch.int32, device=DEV)
    ws = torch.empty(difr.lmhead_workspace_bytes(N, V, d), dtype=torch.uint8, device=DEV)

    def step():
        return difr.lmhead_score(H, W, 1.0, seeds, sid, pos, cg, cg, workspace=ws)

    def load(seed):
        gg = torch.Generator().manual_seed(seed)
        H.copy_(torch.randn(N, d, generator=gg).to(torch.bfloat16).to(DEV))
        cg.copy_(torch.randint(0, V, (N,), generator=gg, dtype=torch.int32).to(DEV))

    load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = step()
    for rep, seed in enumerate((21, 22, 23)):
        load(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [{k: v.clone() for k, v in dd.items()} for dd in captured]
        ws.fill_(0xAB)                 # the workspace carries nothing from one call to the next
        eager = step()
        torch.cuda.synchronize()
        for d_got, d_eager, name in zip(got, eager, ("gumbel", "ipt")):
            _same(d_got, d_eager, "replay %d %s" % (rep, name))
