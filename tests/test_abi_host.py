"""Host-side checks that need no GPU: the C-ABI library loads, exports every function that
include/difr.h declares, rejects bad arguments before touching the device, and its host Philox
agrees with the published vectors."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "difr.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2511_02620_amd import binding

    if not os.path.exists(binding.lib_path()):
        from paper_2511_02620_amd import build

        build.build(verbose=False)
    return binding.load_library()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(difr_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2511_02620_amd import binding

    names = _declared()
    assert set(names) == set(binding.EXPORTS), names
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings_and_version(lib):
    assert lib.difr_version() >= 100
    seen = set()
    for code in range(0, 9):
        s = lib.difr_status_string(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in lib.difr_status_string(99).decode()


def test_host_philox_known_answers(lib):
    from paper_2511_02620_amd import binding

    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        got = binding.philox4x32_10([int(x, 16) for x in t[0:4]], [int(x, 16) for x in t[4:6]])
        for j, w in enumerate(t[6:10]):
            if set(w) != {"-"}:
                assert got[j] == int(w, 16)


def test_argument_validation_needs_no_device(lib):
    from paper_2511_02620_amd.binding import _Rows

    OK, NULL, SHAPE, DTYPE, TEMP, ALIGN, _, _, ARG = range(9)
    fake = 0x1000                       # never dereferenced: every call below fails validation first

    def rows(**kw):
        r = _Rows()
        r.logits, r.dtype, r.N, r.V, r.ld = fake, 0, 4, 16, 16
        r.temperature, r.temperatures = 1.0, None
        r.seeds, r.S, r.seq_ids, r.positions, r.claimed = fake, 1, fake, fake, fake
        for k, v in kw.items():
            setattr(r, k, v)
        return r

    def g(r, margin=fake, argmax=fake, flags=fake):
        return lib.difr_gumbel_score(C.byref(r), margin, argmax, None, None, flags, None, None)

    def i(r, dist=fake, flags=fake, sigma=0.01, eps=1e-30, log_mass=None):
        return lib.difr_ipt_score(C.byref(r), dist, None, None, None, None, sigma, eps, log_mass, flags, None, None)

    def both(r, margin=fake, argmax=fake, fg=fake, dist=fake, fi=fake, sigma=0.01, lm=None):
        return lib.difr_score_both(C.byref(r), fake, margin, argmax, None, None, fg, None, dist, None, None, None, None,
                                   sigma, 1e-30, lm, fi, None)

    assert lib.difr_gumbel_score(None, fake, fake, None, None, fake, None, None) == NULL
    assert lib.difr_score_both(None, fake, fake, fake, None, None, fake, None, fake, None, None, None, None, 0.01, 1e-30,
                               None, fake, None) == NULL
    assert both(rows(), sigma=0.0, lm=fake) == ARG and both(rows(), sigma=float("nan"), lm=fake) == ARG
    for bad, want in ((rows(N=-1), SHAPE), (rows(V=0), SHAPE), (rows(ld=15), SHAPE), (rows(S=0), SHAPE),
                      (rows(N=1 << 31), SHAPE), (rows(V=1 << 31, ld=1 << 31), SHAPE), (rows(dtype=2), DTYPE),
                      (rows(temperature=0.0), TEMP), (rows(temperature=-1.0), TEMP),
                      (rows(temperature=float("nan")), TEMP), (rows(temperature=float("inf")), TEMP),
                      (rows(logits=None), NULL), (rows(seeds=None), NULL), (rows(seq_ids=None), NULL),
                      (rows(positions=None), NULL), (rows(logits=0x1001), ALIGN), (rows(dtype=1, logits=0x1002), ALIGN)):
        assert g(bad) == want, want
        assert i(bad) == want, want
        if want != ALIGN:   # unaligned rows are served by the generic kernels
            assert both(bad) == want, want
    assert g(rows(), margin=None) == NULL and g(rows(), argmax=None) == NULL and g(rows(), flags=None) == NULL
    assert i(rows(), dist=None) == NULL and i(rows(), flags=None) == NULL
    for kw in ("margin", "argmax", "fg", "dist", "fi"):
        assert both(rows(), **{kw: None}) == NULL, kw
    assert both(rows(N=0)) == OK
    assert i(rows(), sigma=0.0, log_mass=fake) == ARG and i(rows(), eps=-1.0, log_mass=fake) == ARG
    # an empty batch is a successful no-op and needs nothing else
    assert g(rows(N=0, logits=None, seeds=None)) == OK and i(rows(N=0)) == OK
    # pooling
    assert lib.difr_seq_reduce(fake, None, fake, -1, 1, 0.0, None, None, None, None, None) == SHAPE
    assert lib.difr_seq_reduce(fake, None, None, 4, 1, 0.0, None, None, None, None, None) == NULL
    assert lib.difr_seq_reduce(None, None, fake, 4, 1, 0.0, None, None, None, None, None) == NULL
    assert lib.difr_seq_reduce(fake, None, fake, 4, 1, float("nan"), None, None, None, None, None) == ARG
    assert lib.difr_seq_reduce(None, None, None, 0, 0, 0.0, None, None, None, None, None) == OK
    # classification
    assert lib.difr_classify(fake, fake, -1, 0.0, 8, 100, None, fake, None, None) == SHAPE
    assert lib.difr_classify(fake, fake, 4, 0.0, 8, 0, None, fake, None, None) == SHAPE
    assert lib.difr_classify(None, fake, 4, 0.0, 8, 100, None, fake, None, None) == NULL
    assert lib.difr_classify(fake, None, 4, 0.0, 8, 100, None, fake, None, None) == NULL
    assert lib.difr_classify(fake, fake, 4, 0.0, 8, 100, None, None, None, None) == NULL
    assert lib.difr_classify(fake, fake, 4, float("nan"), 8, 100, None, fake, None, None) == ARG
    assert lib.difr_classify(None, None, 0, 0.0, 8, 100, None, None, None, None) == OK
    # filtered IPT
    def iptf(r=None, k=50, p=0.95, dist=fake, fl=fake, sigma=0.01, lm=None):
        return lib.difr_ipt_score_filtered(C.byref(r or rows()), k, p, dist, None, None, None, None, sigma,
                                           1e-30, lm, None, fl, None)

    assert iptf(k=-1) == ARG and iptf(k=257) == ARG and iptf(p=0.0) == ARG and iptf(sigma=0.0, lm=fake) == ARG
    assert iptf(k=0, p=1.0) == ARG                            # no filter at all is difr_ipt_score
    assert iptf(rows(V=15, ld=15), k=0, p=0.9) == ALIGN and iptf(rows(N=0), k=0, p=0.9, dist=None, fl=None) == OK
    assert iptf(dist=None) == NULL and iptf(fl=None) == NULL
    assert iptf(rows(V=15, ld=15)) == ALIGN and iptf(rows(N=0), dist=None, fl=None) == OK
    # likelihood estimate
    from paper_2511_02620_amd.binding import _LikelihoodParams

    def lik(r=None, pi=fake, fl=fake, **kw):
        prm = dict(top_k=50, top_p=0.95, s=16, sigma=0.5, M=64, z=fake)
        prm.update(kw)
        p = _LikelihoodParams(prm["top_k"], prm["top_p"], prm["s"], prm["sigma"], prm["M"], prm["z"])
        return lib.difr_gumbel_likelihood(C.byref(r or rows()), C.byref(p), pi, None, None, None, fl, None)

    for kw in (dict(s=-1), dict(s=257), dict(top_k=-1), dict(top_k=257), dict(M=0), dict(sigma=0.0),
               dict(sigma=float("nan")), dict(top_p=0.0)):
        assert lik(**kw) == ARG, kw
    assert lik(top_k=0, top_p=0.9) == NULL                   # the tau output is required then (it carries the nucleus' threshold)
    assert lik(z=None) == NULL and lik(pi=None) == NULL and lik(fl=None) == NULL
    assert lik(rows(V=0)) == SHAPE and lik(rows(N=0), pi=None, fl=None, z=None) == OK
    assert lik(rows(V=15, ld=15)) == ALIGN                   # rows not 16-byte aligned
    assert lib.difr_gumbel_likelihood(C.byref(rows()), None, fake, None, None, None, fake, None) == NULL
    # likelihood + filtered IPT in one pass
    def sbf(r=None, pi=fake, dist=fake, fg=fake, fi=fake, lm=None, sigma_ipt=0.01, **kw):
        prm = dict(top_k=50, top_p=0.95, s=16, sigma=0.5, M=64, z=fake)
        prm.update(kw)
        p = _LikelihoodParams(prm["top_k"], prm["top_p"], prm["s"], prm["sigma"], prm["M"], prm["z"])
        return lib.difr_score_both_filtered(C.byref(r or rows()), None, C.byref(p), pi, None, None, None, fg, dist, None,
                                            None, None, None, sigma_ipt, 1e-30, lm, None, fi, None)

    for kw in (dict(s=-1), dict(s=257), dict(top_k=-1), dict(top_k=257), dict(M=0), dict(sigma=0.0), dict(top_p=0.0)):
        assert sbf(**kw) == ARG, kw
    assert sbf(lm=fake, sigma_ipt=0.0) == ARG
    assert sbf(top_k=0) == NULL                              # a bare nucleus needs the tau array
    assert sbf(top_k=0, top_p=1.0) == ARG                    # ... and no filter at all is not this call
    assert sbf(pi=None) == NULL and sbf(dist=None) == NULL and sbf(fg=None) == NULL and sbf(fi=None) == NULL
    assert sbf(z=None) == NULL and sbf(rows(V=15, ld=15)) == ALIGN and sbf(rows(V=0)) == SHAPE
    assert sbf(rows(N=0), pi=None, dist=None, fg=None, fi=None, z=None) == OK
    # both estimators + admissible-set size in one pass
    def sba(r=None, delta=1.0, margin=fake, count=fake):
        return lib.difr_score_both_admissible(C.byref(r or rows()), None, C.c_float(delta), margin, fake, None, None, fake,
                                              fake, None, None, None, fake, count, None, None)

    assert sba(delta=-1.0) == ARG and sba(delta=float("inf")) == ARG and sba(delta=float("nan")) == ARG
    assert sba(margin=None) == NULL and sba(count=None) == NULL
    assert sba(rows(V=15, ld=15)) == ALIGN and sba(rows(V=0)) == SHAPE and sba(rows(N=0), margin=None, count=None) == OK
    # admissible-set size
    assert lib.difr_admissible_count(C.byref(rows()), fake, C.c_float(-1.0), fake, None, None) == ARG
    assert lib.difr_admissible_count(C.byref(rows()), fake, C.c_float(float("nan")), fake, None, None) == ARG
    assert lib.difr_admissible_count(C.byref(rows()), None, C.c_float(1.0), fake, None, None) == NULL
    assert lib.difr_admissible_count(C.byref(rows()), fake, C.c_float(1.0), None, None, None) == NULL
    assert lib.difr_admissible_count(C.byref(rows(V=0)), fake, C.c_float(1.0), fake, None, None) == SHAPE
    assert lib.difr_admissible_count(C.byref(rows(N=0)), None, C.c_float(1.0), None, None, None) == OK
    # fused LM head
    from paper_2511_02620_amd.binding import _LmHead

    def lm(**kw):
        r = _LmHead()
        r.hidden, r.weight, r.N, r.V, r.d, r.ldh, r.ldw = fake, fake, 4, 100, 128, 128, 128
        r.temperature, r.temperatures = 1.0, None
        r.seeds, r.S, r.seq_ids, r.positions, r.claimed_gumbel, r.claimed_ipt = fake, 1, fake, fake, fake, fake
        for k, v in kw.items():
            setattr(r, k, v)
        return r

    def lms(r, ws=fake, ws_bytes=1 << 20, margin=fake, sigma=0.01, lm_out=None, tok=None):
        return lib.difr_lmhead_score(C.byref(r), margin, fake, None, None, fake, None, fake, None, None, None, tok, sigma,
                                     1e-30, lm_out, fake, ws, ws_bytes, None)

    def lmst(r, margin=fake, sigma=0.01, lm_out=None):
        return lib.difr_lmhead_score_static(C.byref(r), margin, fake, None, None, fake, None, fake, None, None, None, sigma,
                                            1e-30, lm_out, fake, None)

    need = lib.difr_lmhead_workspace_bytes(4, 100, 128, 0)
    assert 0 < need < 1 << 20 and lib.difr_lmhead_workspace_bytes(0, 100, 128, 0) == 0
    assert lib.difr_lmhead_workspace_bytes(16384, 151936, 4096, 0) < 4 << 20
    need_tok = lib.difr_lmhead_workspace_bytes(4, 100, 128, 1)          # one tile: 16 bytes per token more, and 16
    assert need_tok == need + 4 * 16 + 4 * 16
    assert lms(lm(), tok=fake, ws_bytes=need_tok - 1) == SHAPE and lms(lm(), tok=fake, ws_bytes=need_tok) != SHAPE
    for bad, want in ((lm(N=-1), SHAPE), (lm(V=0), SHAPE), (lm(d=0), SHAPE), (lm(d=96, ldh=96, ldw=96), SHAPE),
                      (lm(ldh=64), SHAPE), (lm(ldw=132), SHAPE), (lm(S=0), SHAPE), (lm(N=1 << 31), SHAPE),
                      (lm(ldh=1 << 23), SHAPE), (lm(ldw=1 << 23), SHAPE),
                      (lm(temperature=0.0), TEMP), (lm(hidden=None), NULL), (lm(weight=None), NULL),
                      (lm(seeds=None), NULL), (lm(hidden=0x1008), ALIGN), (lm(weight=0x1004), ALIGN)):
        assert lms(bad) == want, want
    assert lms(lm(), ws=None) == NULL and lms(lm(), margin=None) == NULL
    assert lms(lm(), ws=0x1004) == ALIGN and lms(lm(), ws_bytes=need - 1) == SHAPE
    assert lms(lm(N=0, hidden=None), ws=None) == OK
    assert lms(lm(), sigma=0.0, lm_out=fake) == ARG and lms(lm(), sigma=0.0) != ARG
    assert lib.difr_lmhead_score(None, fake, fake, None, None, fake, None, fake, None, None, None, None, 0.01, 1e-30, None,
                                 fake, fake, 64, None) == NULL
    # the variant with the built-in buffer: same validation, and a batch beyond its 4 MiB is refused on the host
    assert lmst(lm(N=-1)) == SHAPE and lmst(lm(hidden=None)) == NULL and lmst(lm(), margin=None) == NULL
    assert lmst(lm(), sigma=0.0, lm_out=fake) == ARG and lmst(lm(N=0, hidden=None)) == OK
    assert lmst(lm(N=120000)) == 9 and b"built-in" in lib.difr_status_string(9)
    assert lib.difr_debug_noise(C.byref(rows()), 4, 0, fake, None) == SHAPE
    assert lib.difr_debug_gumbel_map(None, 4, fake, None) == NULL


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    from paper_2511_02620_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libdifr.so"))
    with pytest.raises(ImportError):
        binding.load_library()
