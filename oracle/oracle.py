"""ctypes front of the C++ oracle (oracle/intsgd_oracle.cpp): numpy in, numpy out.

Test infrastructure only.  Every function takes the slice start ``j0`` (global
index of the first coordinate of the arrays handed in), so any window of a large
vector can be checked on its own.  Rounding: 0 = nearest-even (Section 5.1),
1 = randomized Int of Section 2.
"""
import ctypes as C

import numpy as np

from . import build as _build

__all__ = [
    "philox4x32_10", "random_word", "int_random", "int_nearest", "saturate", "compress",
    "int_sum", "decode_update", "update_norm", "next_alpha", "step", "decode_update_momentum",
    "step_momentum", "diana_compress", "diana_update", "diana_step",
    "max_abs", "heuristic_alpha", "max_abs_sum",
    "ROUND_NEAREST_EVEN", "ROUND_STOCHASTIC",
]

ROUND_NEAREST_EVEN = 0
ROUND_STOCHASTIC = 1

import os as _os

# INTSGD_ORACLE_LIBRARY names another build of the same source (a sanitizer build in the tests)
_lib = C.CDLL(_os.environ.get("INTSGD_ORACLE_LIBRARY") or _build.build())

_u32p = C.POINTER(C.c_uint32)
_u64p = C.POINTER(C.c_uint64)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)

_lib.oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
_lib.oracle_philox4x32_10.restype = None
_lib.oracle_random_word.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
_lib.oracle_random_word.restype = C.c_uint32
_lib.oracle_int_random.argtypes = [C.c_float, C.c_uint32]
_lib.oracle_int_random.restype = C.c_float
_lib.oracle_int_nearest.argtypes = [C.c_float]
_lib.oracle_int_nearest.restype = C.c_float
_lib.oracle_saturate.argtypes = [C.c_float, C.c_int32, C.POINTER(C.c_int)]
_lib.oracle_saturate.restype = C.c_int32
_lib.oracle_compress.argtypes = [_f32p, C.c_uint64, C.c_uint64, _f32p, _u64p, C.c_uint32,
                                 C.c_int, C.c_int32, C.c_uint64, C.c_uint32, C.c_uint32, _i32p]
_lib.oracle_compress.restype = C.c_uint64
_lib.oracle_int_sum.argtypes = [C.POINTER(_i32p), C.c_uint32, C.c_uint64, _i32p]
_lib.oracle_int_sum.restype = C.c_uint64
_lib.oracle_decode_update.argtypes = [_i32p, C.c_uint64, C.c_uint64, _f32p, _u64p, C.c_uint32,
                                      C.c_uint32, C.c_double, _f32p, _f32p, _f32p]
_lib.oracle_decode_update.restype = None
_lib.oracle_decode_update_momentum.argtypes = [_i32p, C.c_uint64, C.c_uint64, _f32p, _u64p,
                                               C.c_uint32, C.c_uint32, C.c_double, C.c_double,
                                               C.c_double, _f32p, _f32p, _f32p, _f32p]
_lib.oracle_decode_update_momentum.restype = None
_lib.oracle_step_momentum.argtypes = [C.POINTER(_f32p), C.c_uint32, C.c_uint64, C.c_uint64, _f32p,
                                      _u64p, C.c_uint32, C.c_int, C.c_int32, C.c_uint64, C.c_uint32,
                                      C.c_double, C.c_double, C.c_double, _f32p, _f32p, _f32p, _f32p,
                                      _i32p, _u64p, _f64p]
_lib.oracle_step_momentum.restype = C.c_uint64
_lib.oracle_diana_compress.argtypes = [_f32p, _f32p, C.c_uint64, C.c_uint64, _f32p, _u64p, C.c_uint32,
                                       C.c_int, C.c_int32, C.c_uint64, C.c_uint32, C.c_uint32,
                                       _i32p, _f32p]
_lib.oracle_diana_compress.restype = C.c_uint64
_lib.oracle_diana_update.argtypes = [_i32p, C.c_uint64, C.c_uint64, _f32p, _u64p, C.c_uint32,
                                     C.c_uint32, C.c_double, _f32p, _f32p, _f32p, _f32p]
_lib.oracle_diana_update.restype = None
_lib.oracle_diana_step.argtypes = [C.POINTER(_f32p), C.POINTER(_f32p), C.c_uint32, C.c_uint64,
                                   C.c_uint64, _f32p, _u64p, C.c_uint32, C.c_int, C.c_int32,
                                   C.c_uint64, C.c_uint32, C.c_double, _f32p, _f32p, _f32p, _f32p,
                                   C.POINTER(_f32p), _i32p, _u64p, _f64p]
_lib.oracle_diana_step.restype = C.c_uint64
_lib.oracle_max_abs.argtypes = [_f32p, C.c_uint64, C.c_uint64, _u64p, C.c_uint32, _f32p]
_lib.oracle_max_abs.restype = None
_lib.oracle_max_abs_sum.argtypes = [C.POINTER(C.c_int32), C.c_uint64, C.c_uint64, _u64p, C.c_uint32,
                                    C.POINTER(C.c_uint32)]
_lib.oracle_max_abs_sum.restype = None
_lib.oracle_heuristic_alpha.argtypes = [_f32p, C.c_uint32, C.c_uint32, C.c_uint32, _f64p, _f32p]
_lib.oracle_heuristic_alpha.restype = None
_lib.oracle_update_norm.argtypes = [_f32p, _f32p, C.c_uint64, C.c_uint64, _u64p, C.c_uint32,
                                    _f64p]
_lib.oracle_update_norm.restype = None
_lib.oracle_next_alpha.argtypes = [_f64p, _f64p, C.c_uint32, _u64p, C.c_uint64, C.c_uint32,
                                   C.c_double, C.c_double, C.c_double, _f64p, _f32p]
_lib.oracle_next_alpha.restype = C.c_int
_lib.oracle_step.argtypes = [C.POINTER(_f32p), C.c_uint32, C.c_uint64, C.c_uint64, _f32p, _u64p,
                             C.c_uint32, C.c_int, C.c_int32, C.c_uint64, C.c_uint32, C.c_double,
                             _f32p, _f32p, _i32p, _u64p, _f64p]
_lib.oracle_step.restype = C.c_uint64


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _offsets(offsets, B):
    if offsets is None:
        assert B == 1
        return None, None
    off = _arr(offsets, np.uint64)
    assert off.shape == (B + 1,)
    return off, _ptr(off, C.c_uint64)


def _alpha(alpha):
    a = np.atleast_1d(_arr(alpha, np.float32))
    return a, _ptr(a, C.c_float)


def philox4x32_10(counter, key):
    c = _arr(counter, np.uint32)
    k = _arr(key, np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, np.uint32)
    _lib.oracle_philox4x32_10(_ptr(c, C.c_uint32), _ptr(k, C.c_uint32), _ptr(out, C.c_uint32))
    return out


def random_word(seed, step, worker, j):
    return int(_lib.oracle_random_word(int(seed), int(step), int(worker), int(j)))


def int_random(t, word):
    return float(_lib.oracle_int_random(float(np.float32(t)), int(word)))


def int_nearest(t):
    return float(_lib.oracle_int_nearest(float(np.float32(t))))


def saturate(r, L):
    flag = C.c_int(0)
    q = _lib.oracle_saturate(float(np.float32(r)), int(L), C.byref(flag))
    return int(q), int(flag.value)


def compress(g, alpha, *, rounding, L, seed=0, step=0, worker=0, j0=0, offsets=None):
    """Integer message of one worker on a slice -> (q int32[len], clip count)."""
    g = _arr(g, np.float32)
    a, ap = _alpha(alpha)
    off, offp = _offsets(offsets, a.size)
    q = np.empty(g.size, np.int32)
    cnt = _lib.oracle_compress(_ptr(g, C.c_float), int(j0), g.size, ap, offp, a.size,
                               int(rounding), int(L), int(seed), int(step), int(worker),
                               _ptr(q, C.c_int32))
    return q, int(cnt)


def int_sum(qs):
    """Exact sum of n int32 vectors -> (sum int32[len], number of int32 overflows)."""
    qs = [_arr(q, np.int32) for q in qs]
    n, ln = len(qs), qs[0].size
    assert all(q.size == ln for q in qs)
    ptrs = (_i32p * n)(*[_ptr(q, C.c_int32) for q in qs])
    s = np.empty(ln, np.int32)
    ovf = _lib.oracle_int_sum(ptrs, n, ln, _ptr(s, C.c_int32))
    return s, int(ovf)


def decode_update(S, alpha, x, *, n, eta, j0=0, offsets=None, want_gtilde=False):
    S = _arr(S, np.int32)
    x = _arr(x, np.float32)
    assert S.size == x.size
    a, ap = _alpha(alpha)
    off, offp = _offsets(offsets, a.size)
    xn = np.empty_like(x)
    gt = np.empty_like(x) if want_gtilde else None
    _lib.oracle_decode_update(_ptr(S, C.c_int32), int(j0), S.size, ap, offp, a.size, int(n),
                              float(eta), _ptr(x, C.c_float), _ptr(xn, C.c_float),
                              _ptr(gt, C.c_float) if want_gtilde else None)
    return (xn, gt) if want_gtilde else xn


def update_norm(x_new, x_old, *, j0=0, offsets=None, B=1, out=None):
    xn = _arr(x_new, np.float32)
    xo = _arr(x_old, np.float32)
    assert xn.size == xo.size
    off, offp = _offsets(offsets, B)
    ns = np.zeros(B, np.float64) if out is None else out
    _lib.oracle_update_norm(_ptr(xn, C.c_float), _ptr(xo, C.c_float), int(j0), xn.size, offp, B,
                            _ptr(ns, C.c_double))
    return ns


def next_alpha(normsq, r, *, d, n, beta, eps, eta, offsets=None):
    """-> (r_new f64[B], alpha f64[B], alpha f32[B], bad flag)."""
    ns = np.atleast_1d(_arr(normsq, np.float64))
    r_new = np.atleast_1d(np.array(r, dtype=np.float64, copy=True))
    B = ns.size
    assert r_new.size == B
    off, offp = _offsets(offsets, B)
    ad = np.empty(B, np.float64)
    af = np.empty(B, np.float32)
    bad = _lib.oracle_next_alpha(_ptr(ns, C.c_double), _ptr(r_new, C.c_double), B, offp, int(d),
                                 int(n), float(beta), float(eps), float(eta),
                                 _ptr(ad, C.c_double), _ptr(af, C.c_float))
    return r_new, ad, af, int(bad)


def step(grads, alpha, x, *, rounding, L, eta, seed=0, step=0, j0=0, offsets=None,
         normsq=None):
    """One whole IntSGD step on a slice.

    -> dict(x_new, S, sat_count[n], normsq[B] (accumulated into ``normsq`` if given),
    overflow).
    """
    gs = [_arr(g, np.float32) for g in grads]
    n, ln = len(gs), gs[0].size
    assert all(g.size == ln for g in gs)
    x = _arr(x, np.float32)
    assert x.size == ln
    a, ap = _alpha(alpha)
    B = a.size
    off, offp = _offsets(offsets, B)
    ptrs = (_f32p * n)(*[_ptr(g, C.c_float) for g in gs])
    xn = np.empty_like(x)
    S = np.empty(ln, np.int32)
    sat = np.zeros(n, np.uint64)
    ns = np.zeros(B, np.float64) if normsq is None else normsq
    ovf = _lib.oracle_step(ptrs, n, int(j0), ln, ap, offp, B, int(rounding), int(L), int(seed),
                           int(step), float(eta), _ptr(x, C.c_float), _ptr(xn, C.c_float),
                           _ptr(S, C.c_int32), _ptr(sat, C.c_uint64), _ptr(ns, C.c_double))
    return dict(x_new=xn, S=S, sat_count=sat, normsq=ns, overflow=int(ovf))


def decode_update_momentum(S, alpha, x, m, *, n, eta, mu, wd, j0=0, offsets=None):
    """Momentum / weight-decay update -> (x_new, m_new)."""
    S = _arr(S, np.int32)
    x = _arr(x, np.float32)
    m = _arr(m, np.float32)
    assert S.size == x.size == m.size
    a, ap = _alpha(alpha)
    off, offp = _offsets(offsets, a.size)
    xn = np.empty_like(x)
    mn = np.empty_like(m)
    _lib.oracle_decode_update_momentum(_ptr(S, C.c_int32), int(j0), S.size, ap, offp, a.size,
                                       int(n), float(eta), float(mu), float(wd),
                                       _ptr(x, C.c_float), _ptr(m, C.c_float), _ptr(xn, C.c_float),
                                       _ptr(mn, C.c_float))
    return xn, mn


def step_momentum(grads, alpha, x, m, *, rounding, L, eta, mu, wd, seed=0, step=0, j0=0,
                  offsets=None, normsq=None):
    """One whole step with the momentum / weight-decay update on a slice."""
    gs = [_arr(g, np.float32) for g in grads]
    n, ln = len(gs), gs[0].size
    x = _arr(x, np.float32)
    m = _arr(m, np.float32)
    assert x.size == ln and m.size == ln
    a, ap = _alpha(alpha)
    B = a.size
    off, offp = _offsets(offsets, B)
    ptrs = (_f32p * n)(*[_ptr(g, C.c_float) for g in gs])
    xn = np.empty_like(x)
    mn = np.empty_like(m)
    S = np.empty(ln, np.int32)
    sat = np.zeros(n, np.uint64)
    ns = np.zeros(B, np.float64) if normsq is None else normsq
    ovf = _lib.oracle_step_momentum(ptrs, n, int(j0), ln, ap, offp, B, int(rounding), int(L),
                                    int(seed), int(step), float(eta), float(mu), float(wd),
                                    _ptr(x, C.c_float), _ptr(m, C.c_float), _ptr(xn, C.c_float),
                                    _ptr(mn, C.c_float), _ptr(S, C.c_int32), _ptr(sat, C.c_uint64),
                                    _ptr(ns, C.c_double))
    return dict(x_new=xn, m_new=mn, S=S, sat_count=sat, normsq=ns, overflow=int(ovf))


def diana_compress(g, h_local, alpha, *, rounding, L, seed=0, step=0, worker=0, j0=0, offsets=None):
    """IntDIANA worker side -> (q int32[len], h_local_new, clip count)."""
    g = _arr(g, np.float32)
    hl = _arr(h_local, np.float32)
    assert g.size == hl.size
    a, ap = _alpha(alpha)
    off, offp = _offsets(offsets, a.size)
    q = np.empty(g.size, np.int32)
    hn = np.empty_like(hl)
    cnt = _lib.oracle_diana_compress(_ptr(g, C.c_float), _ptr(hl, C.c_float), int(j0), g.size, ap,
                                     offp, a.size, int(rounding), int(L), int(seed), int(step),
                                     int(worker), _ptr(q, C.c_int32), _ptr(hn, C.c_float))
    return q, hn, int(cnt)


def diana_update(S, alpha, x, h, *, n, eta, j0=0, offsets=None):
    """IntDIANA after aggregation -> (x_new, h_new)."""
    S = _arr(S, np.int32)
    x = _arr(x, np.float32)
    h = _arr(h, np.float32)
    a, ap = _alpha(alpha)
    off, offp = _offsets(offsets, a.size)
    xn = np.empty_like(x)
    hn = np.empty_like(h)
    _lib.oracle_diana_update(_ptr(S, C.c_int32), int(j0), S.size, ap, offp, a.size, int(n),
                             float(eta), _ptr(x, C.c_float), _ptr(h, C.c_float),
                             _ptr(xn, C.c_float), _ptr(hn, C.c_float))
    return xn, hn


def diana_step(grads, h_local, alpha, x, h, *, rounding, L, eta, seed=0, step=0, j0=0,
               offsets=None, normsq=None):
    """One whole IntDIANA step on a slice."""
    gs = [_arr(g, np.float32) for g in grads]
    hs = [_arr(v, np.float32) for v in h_local]
    n, ln = len(gs), gs[0].size
    assert len(hs) == n and all(v.size == ln for v in gs + hs)
    x = _arr(x, np.float32)
    h = _arr(h, np.float32)
    a, ap = _alpha(alpha)
    B = a.size
    off, offp = _offsets(offsets, B)
    gp = (_f32p * n)(*[_ptr(g, C.c_float) for g in gs])
    hp = (_f32p * n)(*[_ptr(v, C.c_float) for v in hs])
    hn_local = [np.empty(ln, np.float32) for _ in range(n)]
    hnp = (_f32p * n)(*[_ptr(v, C.c_float) for v in hn_local])
    xn = np.empty_like(x)
    hn = np.empty_like(h)
    S = np.empty(ln, np.int32)
    sat = np.zeros(n, np.uint64)
    ns = np.zeros(B, np.float64) if normsq is None else normsq
    ovf = _lib.oracle_diana_step(gp, hp, n, int(j0), ln, ap, offp, B, int(rounding), int(L),
                                 int(seed), int(step), float(eta), _ptr(x, C.c_float),
                                 _ptr(h, C.c_float), _ptr(xn, C.c_float), _ptr(hn, C.c_float), hnp,
                                 _ptr(S, C.c_int32), _ptr(sat, C.c_uint64), _ptr(ns, C.c_double))
    return dict(x_new=xn, h_new=hn, h_local_new=hn_local, S=S, sat_count=sat, normsq=ns,
                overflow=int(ovf))


def max_abs(g, *, j0=0, offsets=None, B=1, out=None):
    """Running per-block maximum of |g| over finite entries (accumulated into ``out``)."""
    g = _arr(g, np.float32)
    off, offp = _offsets(offsets, B)
    m = np.zeros(B, np.float32) if out is None else out
    _lib.oracle_max_abs(_ptr(g, C.c_float), int(j0), g.size, offp, B, _ptr(m, C.c_float))
    return m


def max_abs_sum(S, *, j0=0, offsets=None, B=1, out=None):
    """Largest |S_j| per block over a slice of the aggregate (running maximum in ``out``)."""
    S = _arr(S, np.int32)
    off, offp = _offsets(offsets, B)
    m = np.zeros(B, np.uint32) if out is None else out
    _lib.oracle_max_abs_sum(_ptr(S, C.c_int32), int(j0), S.size, offp, B, _ptr(m, C.c_uint32))
    return m


def heuristic_alpha(max_abs_per_block, *, n, nb):
    """Heuristic IntSGD scaling -> (alpha f64[B], alpha f32[B])."""
    m = np.atleast_1d(_arr(max_abs_per_block, np.float32))
    ad = np.empty(m.size, np.float64)
    af = np.empty(m.size, np.float32)
    _lib.oracle_heuristic_alpha(_ptr(m, C.c_float), m.size, int(n), int(nb), _ptr(ad, C.c_double),
                                _ptr(af, C.c_float))
    return ad, af
