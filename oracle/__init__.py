"""CPU oracle for the verifier's per-token scores -- TEST INFRASTRUCTURE ONLY.

A ctypes view of ``difr_oracle.c`` (plain C, IEEE double, one row and one
vocabulary entry at a time).  Only the tests, ``__graft_entry__.smoke()`` and the
benchmark's ``cpu_baseline`` leg may import this package; it shares nothing with
the HIP library and never imports it.

Arrays are numpy.  bf16 logits are passed as ``uint16`` bit patterns, fp32 logits
as ``float32``; both are decoded to their exact real value before any arithmetic.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "difr_oracle.c")
_LIB = os.path.join(_HERE, "libdifr_oracle.so")
_lock = threading.Lock()
_lib = None

DTYPE_BF16 = 0
DTYPE_F32 = 1
FLAG_MATCH = 1
FLAG_INVALID_CLAIM = 2
FLAG_NONFINITE = 4
STREAM_GUMBEL = 0
STREAM_IPT = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math) and return the library path."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + ".tmp.%d" % os.getpid()
            cmd = ["gcc", "-O2", "-std=gnu11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                   "-o", tmp, _SRC, "-lm"]
            subprocess.run(cmd, check=True)
            os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    # DIFR_ORACLE_LIB: a test hook.  tests/test_oracle_pins_have_teeth.py points it at deliberately broken
    # builds of the oracle to show that the pins notice; nothing else sets it.
    lib = C.CDLL(os.environ.get("DIFR_ORACLE_LIB") or build())
    u32p, u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    f32p, f64p, u8p = C.POINTER(C.c_float), C.POINTER(C.c_double), C.POINTER(C.c_uint8)
    lib.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
    lib.oracle_philox4x32_10.restype = None
    lib.oracle_noise_word.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]
    lib.oracle_noise_word.restype = C.c_uint32
    lib.oracle_bits_to_uniform.argtypes = [C.c_uint32]
    lib.oracle_bits_to_uniform.restype = C.c_double
    lib.oracle_uniform_to_gumbel.argtypes = [C.c_double]
    lib.oracle_uniform_to_gumbel.restype = C.c_double
    lib.oracle_gumbel_from_bits_array.argtypes = [u32p, C.c_int64, f64p]
    lib.oracle_gumbel_from_bits_array.restype = None
    lib.oracle_noise_row.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int64, u32p]
    lib.oracle_noise_row.restype = None
    lib.oracle_decode_row.argtypes = [C.c_void_p, C.c_int, C.c_int64, f64p]
    lib.oracle_decode_row.restype = None
    lib.oracle_gumbel_row.argtypes = [f64p, C.c_int64, C.c_double, C.c_uint64, C.c_uint32, C.c_uint32,
                                      C.c_int64, f64p, i32p, f64p, f64p, f64p, u8p, f64p]
    lib.oracle_gumbel_row.restype = None
    lib.oracle_gaussian_log_mass.argtypes = [C.c_double] * 5
    lib.oracle_gaussian_log_mass.restype = C.c_double
    lib.oracle_ipt_row.argtypes = [f64p, C.c_int64, C.c_double, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int64,
                                   C.c_double, C.c_double, f64p, f64p, f64p, f64p, i32p, f64p, f64p, u8p]
    lib.oracle_ipt_row.restype = None
    lib.oracle_num_threads.argtypes = []
    lib.oracle_num_threads.restype = C.c_int
    lib.oracle_set_num_threads.argtypes = [C.c_int]
    lib.oracle_set_num_threads.restype = None
    lib.oracle_gumbel_score.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                        f32p, u64p, i32p, u32p, i32p, f64p, i32p, f64p, f64p, f64p, u8p]
    lib.oracle_gumbel_score.restype = C.c_int
    lib.oracle_ipt_score.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                     f32p, u64p, i32p, u32p, i32p, C.c_double, C.c_double,
                                     f64p, f64p, f64p, f64p, i32p, f64p, f64p, u8p]
    lib.oracle_ipt_score.restype = C.c_int
    lib.oracle_ipt_filtered_score.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                              C.POINTER(C.c_float), C.POINTER(C.c_uint64), i32p,
                                              C.POINTER(C.c_uint32), i32p, C.c_int64, C.c_double, C.c_double,
                                              C.c_double, f64p, f64p, f64p, f64p, i32p, f64p, f64p, i32p, f64p, u8p]
    lib.oracle_ipt_filtered_score.restype = C.c_int
    lib.oracle_likelihood.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                      C.POINTER(C.c_float), C.POINTER(C.c_uint64), i32p, C.POINTER(C.c_uint32), i32p,
                                      C.c_int64, C.c_double, C.c_int64, C.c_double, f64p, C.c_int64,
                                      f64p, f64p, f64p, i32p, f64p, f64p]
    lib.oracle_likelihood.restype = C.c_int
    lib.oracle_admissible_count_row.argtypes = [f64p, C.c_int64, C.c_double, C.c_uint64, C.c_uint32, C.c_uint32,
                                                C.c_double, C.c_double, f64p, i32p, i32p, i32p]
    lib.oracle_admissible_count_row.restype = None
    lib.oracle_admissible_count.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                            C.POINTER(C.c_float), C.POINTER(C.c_uint64), i32p, C.POINTER(C.c_uint32),
                                            C.c_double, C.c_double, i32p, i32p, i32p]
    lib.oracle_admissible_count.restype = C.c_int
    u16p = C.POINTER(C.c_uint16)
    lib.oracle_lmhead_row.argtypes = [u16p, u16p, C.c_int64, C.c_int64, C.c_int64, f64p]
    lib.oracle_lmhead_row.restype = None
    lib.oracle_lmhead_score.argtypes = ([u16p, C.c_int64, u16p, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                         C.c_double, C.POINTER(C.c_float), C.POINTER(C.c_uint64), i32p,
                                         C.POINTER(C.c_uint32), i32p, i32p, C.c_double, C.c_double]
                                        + [f64p, i32p, f64p, f64p, f64p, u8p]
                                        + [f64p, f64p, f64p, f64p, i32p, f64p, f64p, u8p, f64p])
    lib.oracle_lmhead_score.restype = C.c_int
    lib.oracle_logit_rank_row.argtypes = [f64p, C.c_int64, C.c_int64]
    lib.oracle_logit_rank_row.restype = C.c_int32
    lib.oracle_logit_rank.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, i32p, i32p]
    lib.oracle_logit_rank.restype = C.c_int
    lib.oracle_classify.argtypes = [f64p, i32p, C.c_int64, C.c_double, C.c_int64, C.c_int64, f64p, u8p, f64p]
    lib.oracle_classify.restype = None
    lib.oracle_seq_reduce.argtypes = [f64p, u8p, i64p, C.c_int64, C.c_double, f64p, f64p, i32p, u8p]
    lib.oracle_seq_reduce.restype = None
    _lib = lib
    return lib


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _opt(a, dtype, ctype):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, _ptr(a, ctype)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def philox4x32_10(ctr, key):
    """Philox4x32-10 block: 4 counter words, 2 key words -> 4 output words."""
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(c, C.c_uint32), _ptr(k, C.c_uint32), _ptr(out, C.c_uint32))
    return out


def noise_word(seed: int, seq: int, pos: int, stream: int, v: int) -> int:
    return int(_load().oracle_noise_word(int(seed), int(seq), int(pos), int(stream), int(v)))


def noise_row(seed: int, seq: int, pos: int, stream: int, V: int):
    bits = np.zeros(int(V), dtype=np.uint32)
    _load().oracle_noise_row(int(seed), int(seq), int(pos), int(stream), int(V), _ptr(bits, C.c_uint32))
    return bits


def bits_to_uniform(r: int) -> float:
    return float(_load().oracle_bits_to_uniform(int(r)))


def uniform_to_gumbel(u: float) -> float:
    return float(_load().oracle_uniform_to_gumbel(float(u)))


def gumbel_from_bits(bits):
    """bits -> uniform -> Gumbel for an array of raw noise words."""
    b = np.ascontiguousarray(bits, dtype=np.uint32)
    g = np.zeros(b.shape[0], dtype=np.float64)
    _load().oracle_gumbel_from_bits_array(_ptr(b, C.c_uint32), b.shape[0], _ptr(g, C.c_double))
    return g


def gaussian_log_mass(a, b, u, sigma, eps) -> float:
    return float(_load().oracle_gaussian_log_mass(float(a), float(b), float(u), float(sigma), float(eps)))


def _logits_view(logits):
    a = np.asarray(logits)
    if a.dtype == np.uint16:
        dtype = DTYPE_BF16
    elif a.dtype == np.float32:
        dtype = DTYPE_F32
    else:
        raise TypeError("logits must be uint16 (bf16 bit patterns) or float32, got %s" % a.dtype)
    if a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        raise ValueError("logits must be a 2-D row-major array (rows may be padded)")
    return a, dtype, a.strides[0] // a.itemsize


def decode_row(row):
    """Exact double value of every stored logit in one row."""
    a = np.ascontiguousarray(row)
    dtype = DTYPE_BF16 if a.dtype == np.uint16 else DTYPE_F32
    if a.dtype not in (np.uint16, np.float32):
        raise TypeError(a.dtype)
    x = np.zeros(a.shape[0], dtype=np.float64)
    _load().oracle_decode_row(a.ctypes.data, dtype, a.shape[0], _ptr(x, C.c_double))
    return x


def gumbel_row(x, T, seed, seq, pos, claimed, want_scores=False):
    """Token-DiFR for one row of real-valued logits ``x`` (float64)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    V = x.shape[0]
    margin, mx, cs, gap2 = (C.c_double() for _ in range(4))
    am = C.c_int32()
    fl = C.c_uint8()
    y = np.zeros(V, dtype=np.float64) if want_scores else None
    _load().oracle_gumbel_row(_ptr(x, C.c_double), V, float(T), int(seed), int(seq), int(pos), int(claimed),
                              C.byref(margin), C.byref(am), C.byref(mx), C.byref(cs), C.byref(gap2),
                              C.byref(fl), _ptr(y, C.c_double) if want_scores else None)
    out = dict(margin=margin.value, argmax=am.value, max_score=mx.value, claimed_score=cs.value,
               gap2=gap2.value, flags=fl.value)
    if want_scores:
        out["y"] = y
    return out


def ipt_row(x, T, seed, seq, pos, claimed, sigma=0.01, eps=1e-30):
    """Token-IPT-DiFR for one row of real-valued logits ``x`` (float64)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    V = x.shape[0]
    u, a, b, d, lm, edge = (C.c_double() for _ in range(6))
    tok = C.c_int32()
    fl = C.c_uint8()
    _load().oracle_ipt_row(_ptr(x, C.c_double), V, float(T), int(seed), int(seq), int(pos), int(claimed),
                           float(sigma), float(eps), C.byref(u), C.byref(a), C.byref(b), C.byref(d),
                           C.byref(tok), C.byref(lm), C.byref(edge), C.byref(fl))
    return dict(u=u.value, cdf_lo=a.value, cdf_hi=b.value, dist=d.value, ipt_token=tok.value,
                log_mass=lm.value, edge=edge.value, flags=fl.value)


def _aux(N, seeds, seq_ids, positions, claimed, temperatures):
    seeds = np.ascontiguousarray(seeds, dtype=np.uint64)
    seq_ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
    positions = np.ascontiguousarray(positions, dtype=np.uint32)
    assert seq_ids.shape == (N,) and positions.shape == (N,)
    if N:
        assert seq_ids.min() >= 0 and seq_ids.max() < seeds.shape[0]
    claimed, cp = _opt(claimed, np.int32, C.c_int32)
    temperatures, tp = _opt(temperatures, np.float32, C.c_float)
    if claimed is not None:
        assert claimed.shape == (N,)
    if temperatures is not None:
        assert temperatures.shape == (N,)
    return seeds, seq_ids, positions, claimed, cp, temperatures, tp


def gumbel_score(logits, V, temperature, seeds, seq_ids, positions, claimed=None, temperatures=None):
    """Token-DiFR for a batch: logits [N, >=V] (uint16 bf16 bits or float32)."""
    a, dtype, ld = _logits_view(logits)
    N = a.shape[0]
    assert a.shape[1] >= V
    seeds, seq_ids, positions, claimed, cp, temperatures, tp = _aux(N, seeds, seq_ids, positions, claimed,
                                                                    temperatures)
    out = dict(margin=np.zeros(N), argmax=np.zeros(N, np.int32), max_score=np.zeros(N),
               claimed_score=np.zeros(N), gap2=np.zeros(N), flags=np.zeros(N, np.uint8))
    rc = _load().oracle_gumbel_score(a.ctypes.data, dtype, N, int(V), ld, float(temperature), tp,
                                     _ptr(seeds, C.c_uint64), _ptr(seq_ids, C.c_int32),
                                     _ptr(positions, C.c_uint32), cp, _ptr(out["margin"], C.c_double),
                                     _ptr(out["argmax"], C.c_int32), _ptr(out["max_score"], C.c_double),
                                     _ptr(out["claimed_score"], C.c_double), _ptr(out["gap2"], C.c_double),
                                     _ptr(out["flags"], C.c_uint8))
    if rc:
        raise MemoryError("oracle_gumbel_score")
    return out


def ipt_score(logits, V, temperature, seeds, seq_ids, positions, claimed=None, temperatures=None,
              sigma=0.01, eps=1e-30):
    """Token-IPT-DiFR for a batch: logits [N, >=V] (uint16 bf16 bits or float32)."""
    a, dtype, ld = _logits_view(logits)
    N = a.shape[0]
    assert a.shape[1] >= V
    seeds, seq_ids, positions, claimed, cp, temperatures, tp = _aux(N, seeds, seq_ids, positions, claimed,
                                                                    temperatures)
    out = dict(u=np.zeros(N), cdf_lo=np.zeros(N), cdf_hi=np.zeros(N), dist=np.zeros(N),
               ipt_token=np.zeros(N, np.int32), log_mass=np.zeros(N), edge=np.zeros(N),
               flags=np.zeros(N, np.uint8))
    rc = _load().oracle_ipt_score(a.ctypes.data, dtype, N, int(V), ld, float(temperature), tp,
                                  _ptr(seeds, C.c_uint64), _ptr(seq_ids, C.c_int32),
                                  _ptr(positions, C.c_uint32), cp, float(sigma), float(eps),
                                  _ptr(out["u"], C.c_double), _ptr(out["cdf_lo"], C.c_double),
                                  _ptr(out["cdf_hi"], C.c_double), _ptr(out["dist"], C.c_double),
                                  _ptr(out["ipt_token"], C.c_int32), _ptr(out["log_mass"], C.c_double),
                                  _ptr(out["edge"], C.c_double), _ptr(out["flags"], C.c_uint8))
    if rc:
        raise MemoryError("oracle_ipt_score")
    return out


def ipt_filtered_score(logits, V, temperature, seeds, seq_ids, positions, claimed, top_k, top_p, temperatures=None,
                       sigma=0.01, eps=1e-30):
    """Token-IPT-DiFR on the distribution the filtering sampler used (top-k, then top-p renormalised)."""
    a, dtype, ld = _logits_view(logits)
    N = a.shape[0]
    assert a.shape[1] >= V
    seeds, seq_ids, positions, claimed, cp, temperatures, tp = _aux(N, seeds, seq_ids, positions, claimed,
                                                                    temperatures)
    out = dict(u=np.zeros(N), cdf_lo=np.zeros(N), cdf_hi=np.zeros(N), dist=np.zeros(N),
               ipt_token=np.zeros(N, np.int32), log_mass=np.zeros(N), edge=np.zeros(N), kept=np.zeros(N, np.int32),
               gap_p=np.zeros(N), flags=np.zeros(N, np.uint8))
    rc = _load().oracle_ipt_filtered_score(a.ctypes.data, dtype, N, int(V), ld, float(temperature), tp,
                                           _ptr(seeds, C.c_uint64), _ptr(seq_ids, C.c_int32),
                                           _ptr(positions, C.c_uint32), cp, int(top_k), float(top_p), float(sigma),
                                           float(eps), _ptr(out["u"], C.c_double), _ptr(out["cdf_lo"], C.c_double),
                                           _ptr(out["cdf_hi"], C.c_double), _ptr(out["dist"], C.c_double),
                                           _ptr(out["ipt_token"], C.c_int32), _ptr(out["log_mass"], C.c_double),
                                           _ptr(out["edge"], C.c_double), _ptr(out["kept"], C.c_int32),
                                           _ptr(out["gap_p"], C.c_double), _ptr(out["flags"], C.c_uint8))
    if rc:
        raise MemoryError("oracle_ipt_filtered_score")
    return out


def likelihood(logits, V, temperature, seeds, seq_ids, positions, claimed, top_k, top_p, s, sigma, z,
               temperatures=None):
    """Token-DiFR likelihood estimate per row.  z: the standard normal draws (float64 [M]).
    Returns dict(pi, log_pi, tau, active [N, s], gap_s, gap_p)."""
    a, dtype, ld = _logits_view(logits)
    N = a.shape[0]
    assert a.shape[1] >= V
    seeds, seq_ids, positions, claimed, cp, temperatures, tp = _aux(N, seeds, seq_ids, positions, claimed,
                                                                    temperatures)
    z = np.ascontiguousarray(z, dtype=np.float64)
    s = int(s)
    out = dict(pi=np.zeros(N), log_pi=np.zeros(N), tau=np.zeros(N), active=np.full((N, max(s, 1)), -1, np.int32),
               gap_s=np.zeros(N), gap_p=np.zeros(N))
    rc = _load().oracle_likelihood(a.ctypes.data, dtype, N, int(V), ld, float(temperature), tp,
                                   _ptr(seeds, C.c_uint64), _ptr(seq_ids, C.c_int32), _ptr(positions, C.c_uint32),
                                   cp, int(top_k), float(top_p), s, float(sigma), _ptr(z, C.c_double), z.shape[0],
                                   _ptr(out["pi"], C.c_double), _ptr(out["log_pi"], C.c_double),
                                   _ptr(out["tau"], C.c_double), _ptr(out["active"], C.c_int32),
                                   _ptr(out["gap_s"], C.c_double), _ptr(out["gap_p"], C.c_double))
    if rc:
        raise MemoryError("oracle_likelihood")
    out["active"] = out["active"][:, :s]
    return out


def admissible_count_row(x, T, seed, seq, pos, delta, tol=0.0):
    """(count, count at delta - tol, count at delta + tol) of { v : max y - y_v <= delta } for one row of doubles."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.zeros_like(x)
    c, lo, hi = C.c_int32(), C.c_int32(), C.c_int32()
    _load().oracle_admissible_count_row(_ptr(x, C.c_double), x.shape[0], float(T), int(seed), int(seq), int(pos),
                                        float(delta), float(tol), _ptr(y, C.c_double), C.byref(c), C.byref(lo),
                                        C.byref(hi))
    return c.value, lo.value, hi.value


def admissible_count(logits, V, temperature, seeds, seq_ids, positions, delta, tol=0.0, temperatures=None):
    """Admissible-set size per row: dict(count, count_lo, count_hi) of int32 [N]."""
    a, dtype, ld = _logits_view(logits)
    N = a.shape[0]
    assert a.shape[1] >= V
    seeds, seq_ids, positions, _, _, temperatures, tp = _aux(N, seeds, seq_ids, positions, None, temperatures)
    out = dict(count=np.zeros(N, np.int32), count_lo=np.zeros(N, np.int32), count_hi=np.zeros(N, np.int32))
    rc = _load().oracle_admissible_count(a.ctypes.data, dtype, N, int(V), ld, float(temperature), tp,
                                         _ptr(seeds, C.c_uint64), _ptr(seq_ids, C.c_int32),
                                         _ptr(positions, C.c_uint32), float(delta), float(tol),
                                         _ptr(out["count"], C.c_int32), _ptr(out["count_lo"], C.c_int32),
                                         _ptr(out["count_hi"], C.c_int32))
    if rc:
        raise MemoryError("oracle_admissible_count")
    return out


def lmhead_row(h, W):
    """Logits of one position: h [d] and W [V, d] as bf16 bit patterns (uint16); returns float64 [V]."""
    h = np.ascontiguousarray(h, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.uint16)
    V, d = W.shape
    assert h.shape == (d,)
    x = np.zeros(V)
    _load().oracle_lmhead_row(_ptr(h, C.c_uint16), _ptr(W, C.c_uint16), V, d, d, _ptr(x, C.c_double))
    return x


def lmhead_score(hidden, weight, temperature, seeds, seq_ids, positions, claimed_gumbel=None, claimed_ipt=None,
                 temperatures=None, sigma=0.01, eps=1e-30, want_logits=False):
    """Both estimators on logits = hidden @ weight.T (bf16 bit patterns, uint16; [N, d] and [V, d]).
    Returns (gumbel dict, ipt dict[, logits float64 [N, V]])."""
    hidden = np.ascontiguousarray(hidden, dtype=np.uint16)
    weight = np.ascontiguousarray(weight, dtype=np.uint16)
    N, d = hidden.shape
    V = weight.shape[0]
    assert weight.shape[1] == d
    seeds, seq_ids, positions, cg, cgp, temperatures, tp = _aux(N, seeds, seq_ids, positions, claimed_gumbel,
                                                                temperatures)
    ci = None if claimed_ipt is None else np.ascontiguousarray(claimed_ipt, dtype=np.int32)
    cip = None if ci is None else _ptr(ci, C.c_int32)
    g = dict(margin=np.zeros(N), argmax=np.zeros(N, np.int32), max_score=np.zeros(N), claimed_score=np.zeros(N),
             gap2=np.zeros(N), flags=np.zeros(N, np.uint8))
    i = dict(u=np.zeros(N), cdf_lo=np.zeros(N), cdf_hi=np.zeros(N), dist=np.zeros(N),
             ipt_token=np.zeros(N, np.int32), log_mass=np.zeros(N), edge=np.zeros(N), flags=np.zeros(N, np.uint8))
    x = np.zeros((N, V)) if want_logits else None
    rc = _load().oracle_lmhead_score(
        _ptr(hidden, C.c_uint16), d, _ptr(weight, C.c_uint16), d, N, V, d, float(temperature), tp,
        _ptr(seeds, C.c_uint64), _ptr(seq_ids, C.c_int32), _ptr(positions, C.c_uint32), cgp, cip,
        float(sigma), float(eps),
        _ptr(g["margin"], C.c_double), _ptr(g["argmax"], C.c_int32), _ptr(g["max_score"], C.c_double),
        _ptr(g["claimed_score"], C.c_double), _ptr(g["gap2"], C.c_double), _ptr(g["flags"], C.c_uint8),
        _ptr(i["u"], C.c_double), _ptr(i["cdf_lo"], C.c_double), _ptr(i["cdf_hi"], C.c_double),
        _ptr(i["dist"], C.c_double), _ptr(i["ipt_token"], C.c_int32), _ptr(i["log_mass"], C.c_double),
        _ptr(i["edge"], C.c_double), _ptr(i["flags"], C.c_uint8), None if x is None else _ptr(x, C.c_double))
    if rc:
        raise MemoryError("oracle_lmhead_score")
    return (g, i, x) if want_logits else (g, i)


def logit_rank_row(x, claimed) -> int:
    """Number of logits strictly above the claimed token's (rank 0 = highest); -1 for an invalid claim."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    return int(_load().oracle_logit_rank_row(_ptr(x, C.c_double), x.shape[0], int(claimed)))


def logit_rank(logits, V, claimed):
    a, dtype, ld = _logits_view(logits)
    N = a.shape[0]
    claimed, cp = _opt(claimed, np.int32, C.c_int32)
    rank = np.zeros(N, dtype=np.int32)
    if _load().oracle_logit_rank(a.ctypes.data, dtype, N, int(V), ld, cp, _ptr(rank, C.c_int32)):
        raise MemoryError("oracle_logit_rank")
    return rank


def classify(scores, ranks, tau, R, V, log2_admissible=None):
    """Three-class classification and exfiltratable bits per token: dict(cls uint8, bits float64)."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    ranks = np.ascontiguousarray(ranks, dtype=np.int32)
    N = scores.shape[0]
    assert ranks.shape == (N,)
    la, lap = _opt(log2_admissible, np.float64, C.c_double)
    out = dict(cls=np.zeros(N, np.uint8), bits=np.zeros(N))
    _load().oracle_classify(_ptr(scores, C.c_double), _ptr(ranks, C.c_int32), N, float(tau), int(R), int(V), lap,
                            _ptr(out["cls"], C.c_uint8), _ptr(out["bits"], C.c_double))
    return out


def seq_reduce(scores, row_flags, offsets, tau):
    """Per-sequence mean / max / mismatch count / flag over rows [offsets[s], offsets[s+1])."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    S = offsets.shape[0] - 1
    assert S >= 0 and (S == 0 or offsets[-1] <= scores.shape[0])
    rf, rfp = _opt(row_flags, np.uint8, C.c_uint8)
    out = dict(seq_mean=np.zeros(S), seq_max=np.zeros(S), seq_mismatch=np.zeros(S, np.int32),
               seq_flag=np.zeros(S, np.uint8))
    _load().oracle_seq_reduce(_ptr(scores, C.c_double), rfp, _ptr(offsets, C.c_int64), S, float(tau),
                              _ptr(out["seq_mean"], C.c_double), _ptr(out["seq_max"], C.c_double),
                              _ptr(out["seq_mismatch"], C.c_int32), _ptr(out["seq_flag"], C.c_uint8))
    return out


def calibrate_threshold(honest_means, fpr: float, as_float32: bool = True) -> float:
    """Threshold from benign pooled scores (appendix on score statistics: pick the
    percentile of the benign distribution that meets the target false-positive rate).
    Scores here are suspiciousness, so tau is the ceil((1-fpr)*n)-th smallest benign
    mean: at most floor(fpr*n) benign units lie strictly above it."""
    m = np.sort(np.asarray(honest_means, dtype=np.float64))
    n = m.shape[0]
    if n == 0:
        raise ValueError("no benign scores")
    k = int(np.ceil((1.0 - fpr) * n))
    k = min(max(k, 1), n)
    tau = float(m[k - 1])
    if as_float32:
        # the library's threshold argument is fp32: return the smallest fp32 value that is not
        # below the chosen benign mean, so that mean stays on the unflagged side after rounding
        t32 = np.float32(tau)
        if float(t32) < tau:
            t32 = np.nextafter(t32, np.float32(np.inf))
        tau = float(t32)
    return tau
