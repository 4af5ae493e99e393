"""The entry point for callers that cannot allocate (difr_lmhead_score_static): its outputs must equal
difr_lmhead_score's bit for bit (same kernels, the partial results in the library's built-in buffer instead
of a caller workspace), on two calls in a row, the second with a smaller batch whose partial results lie over
the leftovers of the first; a batch beyond the buffer's size must be refused before anything is launched."""
import ctypes as C
import dataclasses
import sys

import numpy as np
import pytest
import torch

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


def _inputs(S, L, V, d, claims_seed):
    wl = dataclasses.replace(W.C4_LMHEAD, S=S, L=L, V=V, d=d, temperature=0.8, w_sigma=2.0 / d ** 0.5)
    Wm = wl.weight(DEV)
    Hv, _ = wl.hidden(DEV)
    seeds, sid, pos = wl.seeds().to(DEV), wl.seq_ids().to(DEV), wl.positions().to(DEV)
    gen = torch.Generator().manual_seed(claims_seed)
    cg = torch.randint(0, V, (wl.N,), generator=gen, dtype=torch.int32).to(DEV)
    ci = torch.randint(0, V, (wl.N,), generator=gen, dtype=torch.int32).to(DEV)
    return wl, Hv, Wm, seeds, sid, pos, cg, ci


def _same(a, b, what):
    for part_a, part_b, name in ((a[0], b[0], "gumbel"), (a[1], b[1], "ipt")):
        for k in part_a:
            x, y = part_a[k].cpu().numpy(), part_b[k].cpu().numpy()
            assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), "%s: %s.%s differs" % (what, name, k)


def test_static_equals_workspace_twice(difr):
    big = _inputs(3, 200, 5000, 192, 11)     # 600 rows: 3 token blocks (last ragged), 20 tiles (last ragged), 20 ranges
    small = _inputs(1, 100, 777, 64, 12)     # 100 rows: 1 token block, 4 tiles; its partials overwrite the start only
    outs = {}
    for name, (wl, Hv, Wm, seeds, sid, pos, cg, ci) in (("big", big), ("small", small)):
        say("no-alloc case", name, wl.N, wl.V, wl.d)
        outs[name] = difr.lmhead_outputs(wl.N, torch.device(DEV), want_rank=True, want_log_mass=True)
    # honest half: the sampler's own tokens as claims on every other row, so that matches occur too
    for wl, Hv, Wm, seeds, sid, pos, cg, ci in (big, small):
        g0, _ = difr.lmhead_score(Hv, Wm, wl.temperature, seeds, sid, pos, None, None)
        cg[::2] = g0["argmax"][::2]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = {}
    for name, (wl, Hv, Wm, seeds, sid, pos, cg, ci) in (("big", big), ("small", small)):
        got[name] = difr.lmhead_score_static(Hv, Wm, wl.temperature, seeds, sid, pos, cg, ci, out=outs[name])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before, "the binding allocated device memory around the static call"
    for name, (wl, Hv, Wm, seeds, sid, pos, cg, ci) in (("big", big), ("small", small)):
        want = difr.lmhead_score(Hv, Wm, wl.temperature, seeds, sid, pos, cg, ci, want_rank=True, want_log_mass=True)
        torch.cuda.synchronize()
        _same(got[name], want, name)
        f = got[name][0]["flags"].cpu().numpy()
        say("no-alloc", name, "rows", wl.N, "matches", int((f & difr.FLAG_MATCH).sum()))
        assert (f & difr.FLAG_MATCH).sum() >= wl.N // 2 - 2
    # and once more in the other order, the big batch over the small one's leftovers
    wl, Hv, Wm, seeds, sid, pos, cg, ci = big
    again = difr.lmhead_score_static(Hv, Wm, wl.temperature, seeds, sid, pos, cg, ci, want_rank=True, want_log_mass=True)
    torch.cuda.synchronize()
    _same(again, got["big"], "big after small")


def test_static_refuses_what_does_not_fit(difr):
    lib = difr.load_library()
    # 120,000 tokens need 120000 * 48 + 64 bytes > 4 MiB: refused on the host, before any pointer is looked at
    N, V, d = 120000, 4096, 64
    assert difr.lmhead_workspace_bytes(N, V, d) > 4 << 20
    from paper_2511_02620_amd.binding import _LmHead
    r = _LmHead()
    dummy = torch.zeros(16, dtype=torch.uint8, device=DEV)
    p = dummy.data_ptr()
    r.hidden = r.weight = r.seeds = r.seq_ids = r.positions = p
    r.N, r.V, r.d, r.ldh, r.ldw, r.S, r.temperature = N, V, d, d, d, 1, 1.0
    out = C.c_void_p(p)
    rc = lib.difr_lmhead_score_static(C.byref(r), out, out, None, None, out, None, out, None, None, None, 0.01, 1e-30, None,
                                      out, None)
    assert rc == 9, rc
    assert b"built-in" in lib.difr_status_string(rc)
    torch.cuda.synchronize()
    assert int(dummy.sum()) == 0
