"""ctypes binding of libdifr.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, hands their device
pointers and the current HIP stream to the C entry point of the same name, and returns
freshly allocated output tensors.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdifr.so")
_lib = None

FLAG_MATCH = 1
FLAG_INVALID_CLAIM = 2
FLAG_NONFINITE = 4
FLAG_SLOW_PATH = 8

DTYPE_BF16 = 0
DTYPE_F32 = 1


class DifrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().difr_status_string(status).decode()
        super().__init__("%s: difr_status %d (%s)" % (where, status, msg))


class _Rows(C.Structure):
    _fields_ = [
        ("logits", C.c_void_p),
        ("dtype", C.c_int32),
        ("N", C.c_int64),
        ("V", C.c_int64),
        ("ld", C.c_int64),
        ("temperature", C.c_float),
        ("temperatures", C.c_void_p),
        ("seeds", C.c_void_p),
        ("S", C.c_int64),
        ("seq_ids", C.c_void_p),
        ("positions", C.c_void_p),
        ("claimed", C.c_void_p),
    ]


class _LmHead(C.Structure):
    _fields_ = [
        ("hidden", C.c_void_p),
        ("weight", C.c_void_p),
        ("N", C.c_int64),
        ("V", C.c_int64),
        ("d", C.c_int64),
        ("ldh", C.c_int64),
        ("ldw", C.c_int64),
        ("temperature", C.c_float),
        ("temperatures", C.c_void_p),
        ("seeds", C.c_void_p),
        ("S", C.c_int64),
        ("seq_ids", C.c_void_p),
        ("positions", C.c_void_p),
        ("claimed_gumbel", C.c_void_p),
        ("claimed_ipt", C.c_void_p),
    ]


class _LikelihoodParams(C.Structure):
    _fields_ = [("top_k", C.c_int32), ("top_p", C.c_float), ("s", C.c_int32), ("sigma", C.c_float),
                ("M", C.c_int32), ("z", C.c_void_p)]


EXPORTS = ("difr_gumbel_score", "difr_debug_gumbel_score_unfiltered", "difr_ipt_score", "difr_score_both", "difr_score_both_peaked", "difr_score_both_admissible", "difr_admissible_count", "difr_gumbel_likelihood", "difr_ipt_score_filtered", "difr_score_both_filtered", "difr_lmhead_score", "difr_lmhead_score_static", "difr_lmhead_workspace_bytes", "difr_classify", "difr_seq_reduce", "difr_debug_noise", "difr_debug_gumbel_map",
           "difr_philox4x32_10", "difr_status_string", "difr_version")


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libdifr.so.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libdifr.so is missing at %s: build it with `python -m paper_2511_02620_amd.build` "
                          "(there is no CPU fallback)" % _LIB_PATH)
    lib = C.CDLL(_LIB_PATH)
    vp = C.c_void_p
    lib.difr_gumbel_score.argtypes = [C.POINTER(_Rows), vp, vp, vp, vp, vp, vp, vp]
    lib.difr_gumbel_score.restype = C.c_int
    lib.difr_debug_gumbel_score_unfiltered.argtypes = [C.POINTER(_Rows), vp, vp, vp, vp, vp, vp, vp]
    lib.difr_debug_gumbel_score_unfiltered.restype = C.c_int
    lib.difr_ipt_score.argtypes = [C.POINTER(_Rows), vp, vp, vp, vp, vp, C.c_double, C.c_double, vp, vp, vp, vp]
    lib.difr_score_both.argtypes = [C.POINTER(_Rows)] + [vp] * 12 + [C.c_double, C.c_double, vp, vp, vp]
    lib.difr_score_both.restype = C.c_int
    lib.difr_score_both_peaked.argtypes = lib.difr_score_both.argtypes
    lib.difr_score_both_peaked.restype = C.c_int
    lib.difr_score_both_admissible.argtypes = [C.POINTER(_Rows), vp, C.c_float] + [vp] * 13
    lib.difr_score_both_admissible.restype = C.c_int
    lib.difr_ipt_score_filtered.argtypes = [C.POINTER(_Rows), C.c_int32, C.c_float, vp, vp, vp, vp, vp, C.c_double,
                                            C.c_double, vp, vp, vp, vp]
    lib.difr_ipt_score_filtered.restype = C.c_int
    lib.difr_gumbel_likelihood.argtypes = [C.POINTER(_Rows), C.POINTER(_LikelihoodParams), vp, vp, vp, vp, vp, vp]
    lib.difr_gumbel_likelihood.restype = C.c_int
    lib.difr_score_both_filtered.argtypes = [C.POINTER(_Rows), vp, C.POINTER(_LikelihoodParams)] + [vp] * 10 + [
        C.c_double, C.c_double, vp, vp, vp, vp]
    lib.difr_score_both_filtered.restype = C.c_int
    lib.difr_admissible_count.argtypes = [C.POINTER(_Rows), vp, C.c_float, vp, vp, vp]
    lib.difr_admissible_count.restype = C.c_int
    lib.difr_lmhead_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int32]
    lib.difr_lmhead_workspace_bytes.restype = C.c_size_t
    lib.difr_lmhead_score.argtypes = [C.POINTER(_LmHead)] + [vp] * 11 + [C.c_double, C.c_double, vp, vp, vp, C.c_size_t, vp]
    lib.difr_lmhead_score.restype = C.c_int
    lib.difr_lmhead_score_static.argtypes = [C.POINTER(_LmHead)] + [vp] * 10 + [C.c_double, C.c_double, vp, vp, vp]
    lib.difr_lmhead_score_static.restype = C.c_int
    lib.difr_classify.argtypes = [vp, vp, C.c_int64, C.c_float, C.c_int64, C.c_int64, vp, vp, vp, vp]
    lib.difr_classify.restype = C.c_int
    lib.difr_ipt_score.restype = C.c_int
    lib.difr_seq_reduce.argtypes = [vp, vp, vp, C.c_int64, C.c_int64, C.c_float, vp, vp, vp, vp, vp]
    lib.difr_seq_reduce.restype = C.c_int
    lib.difr_debug_noise.argtypes = [C.POINTER(_Rows), C.c_int64, C.c_int32, vp, vp]
    lib.difr_debug_noise.restype = C.c_int
    lib.difr_debug_gumbel_map.argtypes = [vp, C.c_int64, vp, vp]
    lib.difr_debug_gumbel_map.restype = C.c_int
    lib.difr_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    lib.difr_philox4x32_10.restype = None
    lib.difr_status_string.argtypes = [C.c_int]
    lib.difr_status_string.restype = C.c_char_p
    lib.difr_version.argtypes = []
    lib.difr_version.restype = C.c_int
    _lib = lib
    return lib


def version() -> int:
    return int(load_library().difr_version())


def philox4x32_10(ctr, key):
    """Host helper: one Philox4x32-10 block (4 counter words, 2 key words) -> 4 words."""
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    out = (C.c_uint32 * 4)()
    load_library().difr_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def _stream_ptr(device) -> int:
    return int(torch.cuda.current_stream(device).cuda_stream)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _check(t, dtype, n, name, device):
    if t is None:
        return
    if t.device != device:
        raise ValueError("%s must live on %s" % (name, device))
    if t.dtype != dtype or t.dim() != 1 or t.shape[0] != n or not t.is_contiguous():
        raise ValueError("%s must be a contiguous 1-D %s tensor of %d elements" % (name, dtype, n))


def _rows(logits, V, temperature, seeds, seq_ids, positions, claimed, temperatures):
    if not logits.is_cuda:
        raise ValueError("logits must be a GPU tensor")
    if logits.dim() != 2 or logits.stride(1) != 1 and logits.shape[1] > 1:
        raise ValueError("logits must be 2-D with unit column stride")
    if logits.dtype == torch.bfloat16:
        dt = DTYPE_BF16
    elif logits.dtype == torch.float32:
        dt = DTYPE_F32
    else:
        raise ValueError("logits must be bfloat16 or float32")
    dev = logits.device
    N = logits.shape[0]
    V = logits.shape[1] if V is None else int(V)
    ld = logits.stride(0) if N > 1 else max(logits.shape[1], logits.stride(0) if N else 0)
    _check(seq_ids, torch.int32, N, "seq_ids", dev)
    _check(positions, torch.int32, N, "positions", dev)   # uint32 bit patterns held in int32
    _check(claimed, torch.int32, N, "claimed", dev)
    _check(temperatures, torch.float32, N, "temperatures", dev)
    if seeds.device != dev or seeds.dtype != torch.int64 or seeds.dim() != 1 or not seeds.is_contiguous():
        raise ValueError("seeds must be a contiguous 1-D int64 GPU tensor (uint64 bit patterns)")
    r = _Rows()
    r.logits = logits.data_ptr()
    r.dtype = dt
    r.N, r.V, r.ld = N, V, ld
    r.temperature = float(temperature)
    r.temperatures = None if temperatures is None else temperatures.data_ptr()
    r.seeds = seeds.data_ptr()
    r.S = seeds.shape[0]
    r.seq_ids = seq_ids.data_ptr()
    r.positions = positions.data_ptr()
    r.claimed = None if claimed is None else claimed.data_ptr()
    return r, N, dev


def gumbel_score(logits, temperature, seeds, seq_ids, positions, claimed=None, temperatures=None, V=None,
                 want_scores=True, unfiltered=False, want_rank=False):
    """difr_gumbel_score (or, with unfiltered=True, difr_debug_gumbel_score_unfiltered).
    logits [N, >=V] bf16/fp32 on the GPU; seeds int64 [S] (uint64 bits); seq_ids, positions,
    claimed int32 [N].  Returns a dict of device tensors."""
    lib = load_library()
    entry = lib.difr_debug_gumbel_score_unfiltered if unfiltered else lib.difr_gumbel_score
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, claimed, temperatures)
    out = dict(margin=torch.empty(N, dtype=torch.float32, device=dev),
               argmax=torch.empty(N, dtype=torch.int32, device=dev),
               flags=torch.empty(N, dtype=torch.uint8, device=dev))
    if want_scores:
        out["max_score"] = torch.empty(N, dtype=torch.float32, device=dev)
        out["claimed_score"] = torch.empty(N, dtype=torch.float32, device=dev)
    if want_rank:
        out["logit_rank"] = torch.empty(N, dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        rc = entry(C.byref(r), _ptr(out["margin"]), _ptr(out["argmax"]), _ptr(out.get("max_score")),
                                   _ptr(out.get("claimed_score")), _ptr(out["flags"]), _ptr(out.get("logit_rank")),
                                   _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_gumbel_score")
    return out


def ipt_score(logits, temperature, seeds, seq_ids, positions, claimed=None, temperatures=None, V=None,
              want_token=False, want_log_mass=False, sigma=0.01, eps=1e-30, want_interval=True, want_rank=False):
    """difr_ipt_score.  Same inputs as :func:`gumbel_score`.  Returns a dict of device tensors."""
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, claimed, temperatures)
    f32 = dict(dtype=torch.float32, device=dev)
    out = dict(dist=torch.empty(N, **f32), flags=torch.empty(N, dtype=torch.uint8, device=dev))
    if want_interval:
        out.update(cdf_lo=torch.empty(N, **f32), cdf_hi=torch.empty(N, **f32), u=torch.empty(N, **f32))
    if want_token:
        out["ipt_token"] = torch.empty(N, dtype=torch.int32, device=dev)
    if want_log_mass:
        out["log_mass"] = torch.empty(N, **f32)
    if want_rank:
        out["logit_rank"] = torch.empty(N, dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        rc = lib.difr_ipt_score(C.byref(r), _ptr(out["dist"]), _ptr(out.get("cdf_lo")), _ptr(out.get("cdf_hi")),
                                _ptr(out.get("u")), _ptr(out.get("ipt_token")), float(sigma), float(eps),
                                _ptr(out.get("log_mass")), _ptr(out["flags"]), _ptr(out.get("logit_rank")),
                                _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_ipt_score")
    return out


def score_both(logits, temperature, seeds, seq_ids, positions, claimed_gumbel=None, claimed_ipt=None,
               temperatures=None, V=None, want_rank=False, want_token=False, want_log_mass=False, sigma=0.01, eps=1e-30):
    """difr_score_both: both estimators in one pass.  Returns (gumbel dict, ipt dict) of device tensors;
    want_rank adds logit_rank (of the Token-DiFR claim) to the first, want_token / want_log_mass add ipt_token /
    log_mass to the second (as in :func:`ipt_score`)."""
    return _score_both("difr_score_both", logits, temperature, seeds, seq_ids, positions, claimed_gumbel, claimed_ipt,
                       temperatures, V, want_rank, want_token, want_log_mass, sigma, eps)


def score_both_peaked(logits, temperature, seeds, seq_ids, positions, claimed_gumbel=None, claimed_ipt=None,
                      temperatures=None, V=None, want_rank=False, want_token=False, want_log_mass=False, sigma=0.01,
                      eps=1e-30):
    """difr_score_both_peaked: :func:`score_both` for rows known to be concentrated; same arguments, same results."""
    return _score_both("difr_score_both_peaked", logits, temperature, seeds, seq_ids, positions, claimed_gumbel,
                       claimed_ipt, temperatures, V, want_rank, want_token, want_log_mass, sigma, eps)


def _score_both(entry_name, logits, temperature, seeds, seq_ids, positions, claimed_gumbel, claimed_ipt, temperatures, V,
                want_rank, want_token, want_log_mass, sigma, eps):
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, claimed_gumbel, temperatures)
    _check(claimed_ipt, torch.int32, N, "claimed_ipt", dev)
    f32 = dict(dtype=torch.float32, device=dev)
    g = dict(margin=torch.empty(N, **f32), argmax=torch.empty(N, dtype=torch.int32, device=dev),
             max_score=torch.empty(N, **f32), claimed_score=torch.empty(N, **f32),
             flags=torch.empty(N, dtype=torch.uint8, device=dev))
    i = dict(dist=torch.empty(N, **f32), cdf_lo=torch.empty(N, **f32), cdf_hi=torch.empty(N, **f32),
             u=torch.empty(N, **f32), flags=torch.empty(N, dtype=torch.uint8, device=dev))
    if want_rank:
        g["logit_rank"] = torch.empty(N, dtype=torch.int32, device=dev)
    if want_token:
        i["ipt_token"] = torch.empty(N, dtype=torch.int32, device=dev)
    if want_log_mass:
        i["log_mass"] = torch.empty(N, **f32)
    with torch.cuda.device(dev):
        rc = getattr(lib, entry_name)(C.byref(r), _ptr(claimed_ipt), _ptr(g["margin"]), _ptr(g["argmax"]),
                                      _ptr(g["max_score"]), _ptr(g["claimed_score"]), _ptr(g["flags"]),
                                      _ptr(g.get("logit_rank")), _ptr(i["dist"]), _ptr(i["cdf_lo"]), _ptr(i["cdf_hi"]),
                                      _ptr(i["u"]), _ptr(i.get("ipt_token")), float(sigma), float(eps),
                                      _ptr(i.get("log_mass")), _ptr(i["flags"]), _stream_ptr(dev))
    if rc:
        raise DifrError(rc, entry_name)
    return g, i


def score_both_admissible(logits, temperature, seeds, seq_ids, positions, delta, claimed_gumbel=None, claimed_ipt=None,
                          temperatures=None, V=None):
    """difr_score_both_admissible: both estimators and the admissible-set size in one pass.
    Returns (gumbel dict, ipt dict, admissible dict with count [-1 = undetermined] and log2_count)."""
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, claimed_gumbel, temperatures)
    _check(claimed_ipt, torch.int32, N, "claimed_ipt", dev)
    f32 = dict(dtype=torch.float32, device=dev)
    g = dict(margin=torch.empty(N, **f32), argmax=torch.empty(N, dtype=torch.int32, device=dev),
             max_score=torch.empty(N, **f32), claimed_score=torch.empty(N, **f32),
             flags=torch.empty(N, dtype=torch.uint8, device=dev))
    i = dict(dist=torch.empty(N, **f32), cdf_lo=torch.empty(N, **f32), cdf_hi=torch.empty(N, **f32),
             u=torch.empty(N, **f32), flags=torch.empty(N, dtype=torch.uint8, device=dev))
    a = dict(count=torch.empty(N, dtype=torch.int32, device=dev), log2_count=torch.empty(N, **f32))
    with torch.cuda.device(dev):
        rc = lib.difr_score_both_admissible(C.byref(r), _ptr(claimed_ipt), float(delta), _ptr(g["margin"]),
                                            _ptr(g["argmax"]), _ptr(g["max_score"]), _ptr(g["claimed_score"]),
                                            _ptr(g["flags"]), _ptr(i["dist"]), _ptr(i["cdf_lo"]), _ptr(i["cdf_hi"]),
                                            _ptr(i["u"]), _ptr(i["flags"]), _ptr(a["count"]), _ptr(a["log2_count"]),
                                            _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_score_both_admissible")
    return g, i, a


def ipt_score_filtered(logits, temperature, seeds, seq_ids, positions, claimed=None, top_k=50, top_p=1.0,
                       temperatures=None, V=None, want_token=False, want_log_mass=False, sigma=0.01, eps=1e-30):
    """difr_ipt_score_filtered.  Returns a dict of device tensors (dist, cdf_lo, cdf_hi, u, kept, flags, ...)."""
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, claimed, temperatures)
    f32 = dict(dtype=torch.float32, device=dev)
    out = dict(dist=torch.empty(N, **f32), cdf_lo=torch.empty(N, **f32), cdf_hi=torch.empty(N, **f32),
               u=torch.empty(N, **f32), kept=torch.empty(N, dtype=torch.int32, device=dev),
               flags=torch.empty(N, dtype=torch.uint8, device=dev))
    if want_token:
        out["ipt_token"] = torch.empty(N, dtype=torch.int32, device=dev)
    if want_log_mass:
        out["log_mass"] = torch.empty(N, **f32)
    with torch.cuda.device(dev):
        rc = lib.difr_ipt_score_filtered(C.byref(r), int(top_k), float(top_p), _ptr(out["dist"]), _ptr(out["cdf_lo"]),
                                         _ptr(out["cdf_hi"]), _ptr(out["u"]), _ptr(out.get("ipt_token")), float(sigma),
                                         float(eps), _ptr(out.get("log_mass")), _ptr(out["kept"]), _ptr(out["flags"]),
                                         _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_ipt_score_filtered")
    return out


def gumbel_likelihood(logits, temperature, seeds, seq_ids, positions, claimed, z, top_k=0, top_p=1.0, s=16, sigma=1.0,
                      temperatures=None, V=None, want_active=False):
    """difr_gumbel_likelihood.  z: fp32 [M] standard normal draws on the GPU.  Returns a dict of device tensors."""
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, claimed, temperatures)
    if z.device != dev or z.dtype != torch.float32 or z.dim() != 1 or not z.is_contiguous():
        raise ValueError("z must be a contiguous 1-D float32 tensor on the device of logits")
    p = _LikelihoodParams(int(top_k), float(top_p), int(s), float(sigma), z.shape[0], z.data_ptr())
    f32 = dict(dtype=torch.float32, device=dev)
    out = dict(pi=torch.empty(N, **f32), log_pi=torch.empty(N, **f32), tau=torch.empty(N, **f32),
               flags=torch.empty(N, dtype=torch.uint8, device=dev))
    if want_active:
        out["active"] = torch.empty(N, max(int(s), 1), dtype=torch.int32, device=dev)[:, :int(s)].contiguous()
    with torch.cuda.device(dev):
        rc = lib.difr_gumbel_likelihood(C.byref(r), C.byref(p), _ptr(out["pi"]), _ptr(out["log_pi"]), _ptr(out["tau"]),
                                        _ptr(out.get("active")) if int(s) > 0 else None, _ptr(out["flags"]),
                                        _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_gumbel_likelihood")
    return out


def score_both_filtered(logits, temperature, seeds, seq_ids, positions, claimed_gumbel, claimed_ipt, z, top_k=50,
                        top_p=1.0, s=16, sigma=1.0, temperatures=None, V=None, want_active=False, want_token=False,
                        want_log_mass=False, sigma_ipt=0.01, eps=1e-30):
    """difr_score_both_filtered: gumbel_likelihood and ipt_score_filtered in one pass over the logits.
    Returns (likelihood dict, filtered-IPT dict), each as the single call returns it."""
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, claimed_gumbel, temperatures)
    _check(claimed_ipt, torch.int32, N, "claimed_ipt", dev)
    if z.device != dev or z.dtype != torch.float32 or z.dim() != 1 or not z.is_contiguous():
        raise ValueError("z must be a contiguous 1-D float32 tensor on the device of logits")
    p = _LikelihoodParams(int(top_k), float(top_p), int(s), float(sigma), z.shape[0], z.data_ptr())
    f32 = dict(dtype=torch.float32, device=dev)
    lik = dict(pi=torch.empty(N, **f32), log_pi=torch.empty(N, **f32), tau=torch.empty(N, **f32),
               flags=torch.empty(N, dtype=torch.uint8, device=dev))
    if want_active:
        lik["active"] = torch.empty(N, max(int(s), 1), dtype=torch.int32, device=dev)[:, :int(s)].contiguous()
    ipt = dict(dist=torch.empty(N, **f32), cdf_lo=torch.empty(N, **f32), cdf_hi=torch.empty(N, **f32),
               u=torch.empty(N, **f32), kept=torch.empty(N, dtype=torch.int32, device=dev),
               flags=torch.empty(N, dtype=torch.uint8, device=dev))
    if want_token:
        ipt["ipt_token"] = torch.empty(N, dtype=torch.int32, device=dev)
    if want_log_mass:
        ipt["log_mass"] = torch.empty(N, **f32)
    with torch.cuda.device(dev):
        rc = lib.difr_score_both_filtered(C.byref(r), _ptr(claimed_ipt), C.byref(p), _ptr(lik["pi"]), _ptr(lik["log_pi"]),
                                          _ptr(lik["tau"]), _ptr(lik.get("active")) if int(s) > 0 else None,
                                          _ptr(lik["flags"]), _ptr(ipt["dist"]), _ptr(ipt["cdf_lo"]), _ptr(ipt["cdf_hi"]),
                                          _ptr(ipt["u"]), _ptr(ipt.get("ipt_token")), float(sigma_ipt), float(eps),
                                          _ptr(ipt.get("log_mass")), _ptr(ipt["kept"]), _ptr(ipt["flags"]),
                                          _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_score_both_filtered")
    return lik, ipt


def admissible_count(logits, temperature, seeds, seq_ids, positions, max_score, delta, temperatures=None, V=None,
                     want_log2=True):
    """difr_admissible_count: size of { v : max_score - y_v <= delta } per row (max_score from gumbel_score)."""
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, None, temperatures)
    _check(max_score, torch.float32, N, "max_score", dev)
    out = dict(count=torch.empty(N, dtype=torch.int32, device=dev))
    if want_log2:
        out["log2_count"] = torch.empty(N, dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        rc = lib.difr_admissible_count(C.byref(r), _ptr(max_score), float(delta), _ptr(out["count"]),
                                       _ptr(out.get("log2_count")), _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_admissible_count")
    return out


def lmhead_workspace_bytes(N, V, d, want_token=False) -> int:
    return int(load_library().difr_lmhead_workspace_bytes(int(N), int(V), int(d), int(bool(want_token))))


def _lmhead_args(hidden, weight, temperature, seeds, seq_ids, positions, claimed_gumbel, claimed_ipt, temperatures):
    for name, t in (("hidden", hidden), ("weight", weight)):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("%s must be a 2-D bfloat16 GPU tensor with unit column stride" % name)
    dev = hidden.device
    N, d = hidden.shape
    V = weight.shape[0]
    if weight.shape[1] != d or weight.device != dev:
        raise ValueError("weight must be [V, d] on the device of hidden")
    _check(seq_ids, torch.int32, N, "seq_ids", dev)
    _check(positions, torch.int32, N, "positions", dev)
    _check(claimed_gumbel, torch.int32, N, "claimed_gumbel", dev)
    _check(claimed_ipt, torch.int32, N, "claimed_ipt", dev)
    _check(temperatures, torch.float32, N, "temperatures", dev)
    if seeds.device != dev or seeds.dtype != torch.int64 or seeds.dim() != 1 or not seeds.is_contiguous():
        raise ValueError("seeds must be a contiguous 1-D int64 GPU tensor (uint64 bit patterns)")
    r = _LmHead()
    r.hidden, r.weight = hidden.data_ptr(), weight.data_ptr()
    r.N, r.V, r.d = N, V, d
    r.ldh = hidden.stride(0) if N > 1 else d
    r.ldw = weight.stride(0) if V > 1 else d
    r.temperature = float(temperature)
    r.temperatures = None if temperatures is None else temperatures.data_ptr()
    r.seeds, r.S = seeds.data_ptr(), seeds.shape[0]
    r.seq_ids, r.positions = seq_ids.data_ptr(), positions.data_ptr()
    r.claimed_gumbel = None if claimed_gumbel is None else claimed_gumbel.data_ptr()
    r.claimed_ipt = None if claimed_ipt is None else claimed_ipt.data_ptr()
    return r, dev, N, V, d


_LMHEAD_OUT = (("margin", torch.float32), ("argmax", torch.int32), ("max_score", torch.float32),
               ("claimed_score", torch.float32), ("flags", torch.uint8)), (
    ("dist", torch.float32), ("cdf_lo", torch.float32), ("cdf_hi", torch.float32), ("u", torch.float32),
    ("flags", torch.uint8))
_LMHEAD_OPT = (("logit_rank", torch.int32),), (("log_mass", torch.float32), ("ipt_token", torch.int32))


def lmhead_outputs(N, device, want_rank=False, want_log_mass=False, want_token=False):
    """Output buffers of lmhead_score / lmhead_score_static, allocated once and reusable across calls."""
    g, i = tuple({k: torch.empty(N, dtype=dt, device=device) for k, dt in part} for part in _LMHEAD_OUT)
    if want_rank:
        g["logit_rank"] = torch.empty(N, dtype=torch.int32, device=device)
    if want_log_mass:
        i["log_mass"] = torch.empty(N, dtype=torch.float32, device=device)
    if want_token:
        i["ipt_token"] = torch.empty(N, dtype=torch.int32, device=device)
    return g, i


def _lmhead_out(out, N, dev, want_rank, want_log_mass, want_token=False):
    if out is None:
        return lmhead_outputs(N, dev, want_rank, want_log_mass, want_token)
    g, i = out
    for part, spec, opt in zip((g, i), _LMHEAD_OUT, _LMHEAD_OPT):
        for k, dt in spec:
            _check(part[k], dt, N, k, dev)
        for k, dt in opt:
            _check(part.get(k), dt, N, k, dev)
    return g, i


def _lmhead_call(entry_name, token, tail, r, g, i, sigma, eps, dev):
    lib = load_library()
    with torch.cuda.device(dev):
        rc = getattr(lib, entry_name)(C.byref(r), _ptr(g["margin"]), _ptr(g["argmax"]), _ptr(g["max_score"]),
                                      _ptr(g["claimed_score"]), _ptr(g["flags"]), _ptr(g.get("logit_rank")),
                                      _ptr(i["dist"]), _ptr(i["cdf_lo"]), _ptr(i["cdf_hi"]), _ptr(i["u"]), *token,
                                      float(sigma), float(eps), _ptr(i.get("log_mass")), _ptr(i["flags"]), *tail,
                                      _stream_ptr(dev))
    if rc:
        raise DifrError(rc, entry_name)
    return g, i


def lmhead_score(hidden, weight, temperature, seeds, seq_ids, positions, claimed_gumbel=None, claimed_ipt=None,
                 temperatures=None, workspace=None, out=None, want_rank=False, want_log_mass=False, want_token=False,
                 sigma=0.01, eps=1e-30):
    """difr_lmhead_score: both estimators on logits = hidden @ weight.T that are never stored.
    hidden [N, d], weight [V, d] bf16 on the GPU (unit column stride).  Returns (gumbel dict, ipt dict);
    want_rank adds logit_rank (of the Token-DiFR claim) to the first, want_log_mass / want_token add log_mass /
    ipt_token (the sampler's own token; it needs a larger workspace: lmhead_workspace_bytes(..., want_token=True)) to the second;
    `out` = a pair from lmhead_outputs() to write into instead of new tensors (it decides which optional outputs
    are produced)."""
    r, dev, N, V, d = _lmhead_args(hidden, weight, temperature, seeds, seq_ids, positions, claimed_gumbel, claimed_ipt,
                                   temperatures)
    g, i = _lmhead_out(out, N, dev, want_rank, want_log_mass, want_token)
    need = lmhead_workspace_bytes(N, V, d, "ipt_token" in i)
    if workspace is None:
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=dev)
    elif workspace.device != dev or workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 tensor on the device of hidden")
    return _lmhead_call("difr_lmhead_score", (_ptr(i.get("ipt_token")),), (_ptr(workspace), workspace.numel()), r, g, i,
                        sigma, eps, dev)


LMHEAD_STATIC_SCRATCH_BYTES = 4 << 20


def lmhead_score_static(hidden, weight, temperature, seeds, seq_ids, positions, claimed_gumbel=None, claimed_ipt=None,
                        temperatures=None, out=None, want_rank=False, want_log_mass=False, sigma=0.01, eps=1e-30):
    """difr_lmhead_score_static: lmhead_score without a workspace (the library's built-in buffer serves; calls that
    overlap in time on one GPU race on it).  With `out` given (lmhead_outputs()) nothing is allocated at all."""
    r, dev, N, V, d = _lmhead_args(hidden, weight, temperature, seeds, seq_ids, positions, claimed_gumbel, claimed_ipt,
                                   temperatures)
    g, i = _lmhead_out(out, N, dev, want_rank, want_log_mass)
    if "ipt_token" in i:
        raise ValueError("difr_lmhead_score_static has no ipt_token output")
    return _lmhead_call("difr_lmhead_score_static", (), (), r, g, i, sigma, eps, dev)


def seq_reduce(scores, row_flags, seq_offsets, threshold):
    """difr_seq_reduce.  scores fp32 [N], row_flags uint8 [N] or None, seq_offsets int64 [S+1]."""
    lib = load_library()
    if not scores.is_cuda or scores.dtype != torch.float32 or scores.dim() != 1 or not scores.is_contiguous():
        raise ValueError("scores must be a contiguous 1-D float32 GPU tensor")
    dev = scores.device
    N = scores.shape[0]
    _check(row_flags, torch.uint8, N, "row_flags", dev)
    if (seq_offsets.device != dev or seq_offsets.dtype != torch.int64 or seq_offsets.dim() != 1
            or seq_offsets.shape[0] < 1 or not seq_offsets.is_contiguous()):
        raise ValueError("seq_offsets must be a contiguous 1-D int64 GPU tensor of S+1 elements")
    S = seq_offsets.shape[0] - 1
    out = dict(seq_mean=torch.empty(S, dtype=torch.float32, device=dev),
               seq_max=torch.empty(S, dtype=torch.float32, device=dev),
               seq_mismatch=torch.empty(S, dtype=torch.int32, device=dev),
               seq_flag=torch.empty(S, dtype=torch.uint8, device=dev))
    with torch.cuda.device(dev):
        rc = lib.difr_seq_reduce(_ptr(scores), _ptr(row_flags), _ptr(seq_offsets), N, S, float(threshold),
                                 _ptr(out["seq_mean"]), _ptr(out["seq_max"]), _ptr(out["seq_mismatch"]),
                                 _ptr(out["seq_flag"]), _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_seq_reduce")
    return out


def classify(scores, ranks, tau, rank_cutoff, V, log2_admissible=None):
    """difr_classify.  scores fp32 [N], ranks int32 [N] on the GPU.  Returns dict(cls uint8, bits fp32)."""
    lib = load_library()
    if not scores.is_cuda or scores.dtype != torch.float32 or scores.dim() != 1 or not scores.is_contiguous():
        raise ValueError("scores must be a contiguous 1-D float32 GPU tensor")
    dev, N = scores.device, scores.shape[0]
    _check(ranks, torch.int32, N, "ranks", dev)
    _check(log2_admissible, torch.float32, N, "log2_admissible", dev)
    out = dict(cls=torch.empty(N, dtype=torch.uint8, device=dev), bits=torch.empty(N, dtype=torch.float32, device=dev))
    with torch.cuda.device(dev):
        rc = lib.difr_classify(_ptr(scores), _ptr(ranks), N, float(tau), int(rank_cutoff), int(V),
                               _ptr(log2_admissible), _ptr(out["cls"]), _ptr(out["bits"]), _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_classify")
    return out


def debug_noise(logits, temperature, seeds, seq_ids, positions, row, stream, V=None):
    """difr_debug_noise: raw noise words (int32 tensor holding uint32 bits) of one row."""
    lib = load_library()
    r, N, dev = _rows(logits, V, temperature, seeds, seq_ids, positions, None, None)
    bits = torch.empty(int(r.V), dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        rc = lib.difr_debug_noise(C.byref(r), int(row), int(stream), _ptr(bits), _stream_ptr(dev))
    if rc:
        raise DifrError(rc, "difr_debug_noise")
    return bits


def debug_gumbel_map(bits):
    """difr_debug_gumbel_map: device bits -> Gumbel map for an int32 tensor of raw words."""
    lib = load_library()
    if not bits.is_cuda or bits.dtype != torch.int32 or not bits.is_contiguous():
        raise ValueError("bits must be a contiguous int32 GPU tensor")
    g = torch.empty(bits.numel(), dtype=torch.float32, device=bits.device)
    with torch.cuda.device(bits.device):
        rc = lib.difr_debug_gumbel_map(_ptr(bits), bits.numel(), _ptr(g), _stream_ptr(bits.device))
    if rc:
        raise DifrError(rc, "difr_debug_gumbel_map")
    return g
