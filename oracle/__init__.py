"""ctypes front-end of the CPU oracle (test infrastructure only).

Only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the product never does.  All functions take the fp32
arrays that the GPU path gets and return float64 (``long_double=True`` uses the
long-double build and returns ``numpy.longdouble``).  Either ``C`` (dense n x m)
or ``X, Y`` (n x d and m x d points, squared-Euclidean cost) is given.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import build as _build

_libs = {}


def _lib(long_double: bool = False):
    key = bool(long_double)
    if key not in _libs:
        _build.build()
        # FS_ORACLE_LIB: another build of the same source in place of the ordinary one (the sanitizer leg)
        override = os.environ.get("FS_ORACLE_LIB") if not key else None
        lib = ctypes.CDLL(override or (_build.LIB_LD if key else _build.LIB))
        real = ctypes.c_longdouble if key else ctypes.c_double
        lib.fso_marginal_err.restype = real
        lib.fso_solve.restype = ctypes.c_int
        lib.fso_real_bytes.restype = ctypes.c_int
        _libs[key] = lib
    return _libs[key]


def _rdt(long_double):
    return np.longdouble if long_double else np.float64


def _fp(x):
    if x is None:
        return None
    assert x.dtype == np.float32 and x.flags.c_contiguous
    return x.ctypes.data_as(ctypes.c_void_p)


def _rp(x):
    return None if x is None else x.ctypes.data_as(ctypes.c_void_p)


def _geom(C, X, Y, a, b):
    if C is not None:
        assert X is None and Y is None
        n, m = C.shape
        d = 0
    else:
        n, d = X.shape
        m = Y.shape[0]
        assert Y.shape[1] == d
    assert a.shape == (n,) and b.shape == (m,)
    return n, m, d


def _head(C, X, Y, a, b, eps):
    n, m, d = _geom(C, X, Y, a, b)
    return (_fp(C), _fp(X), _fp(Y), ctypes.c_int(d), _fp(a), _fp(b), ctypes.c_int(n), ctypes.c_int(m),
            ctypes.c_double(float(eps))), n, m


def set_threads(k: int) -> None:
    """Set the OpenMP thread count used by subsequent calls (results do not depend on it)."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(k))


def max_threads() -> int:
    omp = ctypes.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def update_f(a, b, eps, g, C=None, X=None, Y=None, long_double=False):
    """One f half-step (Eq. 9) from g."""
    head, n, m = _head(C, X, Y, a, b, eps)
    g = np.ascontiguousarray(g, dtype=_rdt(long_double))
    f = np.empty(n, dtype=_rdt(long_double))
    _lib(long_double).fso_update_f(*head, _rp(g), _rp(f))
    return f


def update_g(a, b, eps, f, C=None, X=None, Y=None, long_double=False):
    """One g half-step (Eq. 10) from f."""
    head, n, m = _head(C, X, Y, a, b, eps)
    f = np.ascontiguousarray(f, dtype=_rdt(long_double))
    g = np.empty(m, dtype=_rdt(long_double))
    _lib(long_double).fso_update_g(*head, _rp(f), _rp(g))
    return g


def marginals(a, b, eps, f, g, C=None, X=None, Y=None, long_double=False):
    """Row and column marginals of the plan, each by its own log-domain LSE (Sec. 4.5)."""
    head, n, m = _head(C, X, Y, a, b, eps)
    dt = _rdt(long_double)
    f = np.ascontiguousarray(f, dtype=dt)
    g = np.ascontiguousarray(g, dtype=dt)
    r, c = np.empty(n, dtype=dt), np.empty(m, dtype=dt)
    _lib(long_double).fso_marginals(*head, _rp(f), _rp(g), _rp(r), _rp(c))
    return r, c


def marginal_err(a, b, eps, f, g, C=None, X=None, Y=None, long_double=False):
    """sum_i |r_i - a_i| (Alg. 1)."""
    head, n, m = _head(C, X, Y, a, b, eps)
    dt = _rdt(long_double)
    f = np.ascontiguousarray(f, dtype=dt)
    g = np.ascontiguousarray(g, dtype=dt)
    return _lib(long_double).fso_marginal_err(*head, _rp(f), _rp(g))


def plan(a, b, eps, f, g, C=None, X=None, Y=None, long_double=False):
    """The n x m plan of Eq. 5."""
    head, n, m = _head(C, X, Y, a, b, eps)
    dt = _rdt(long_double)
    f = np.ascontiguousarray(f, dtype=dt)
    g = np.ascontiguousarray(g, dtype=dt)
    P = np.empty((n, m), dtype=dt)
    _lib(long_double).fso_plan(*head, _rp(f), _rp(g), _rp(P))
    return P


def barycentric(a, b, eps, f, g, Z, C=None, X=None, Y=None, long_double=False):
    """T[i] = sum_j P_ij Z[j] / sum_j P_ij (barycentric mapping, Sec. 5.6); Z is m x dz."""
    head, n, m = _head(C, X, Y, a, b, eps)
    dt = _rdt(long_double)
    f = np.ascontiguousarray(f, dtype=dt)
    g = np.ascontiguousarray(g, dtype=dt)
    Z = np.ascontiguousarray(Z, dtype=dt)
    if Z.ndim != 2 or Z.shape[0] != m:
        raise ValueError("Z must be m x dz")
    T = np.empty((n, Z.shape[1]), dtype=dt)
    _lib(long_double).fso_barycentric(*head, _rp(f), _rp(g), _rp(Z), ctypes.c_int(Z.shape[1]), _rp(T))
    return T


def objectives(a, b, eps, f, g, C=None, X=None, Y=None, long_double=False):
    """dict(cost=<C,P>, mass=sum P, kl=KL(P|a x b), primal=Eq. 3 objective, dual=D(f,g))."""
    head, n, m = _head(C, X, Y, a, b, eps)
    dt = _rdt(long_double)
    f = np.ascontiguousarray(f, dtype=dt)
    g = np.ascontiguousarray(g, dtype=dt)
    out = np.empty(5, dtype=dt)
    _lib(long_double).fso_objectives(*head, _rp(f), _rp(g), _rp(out))
    return dict(cost=out[0], mass=out[1], kl=out[2], primal=out[3], dual=out[4])


def cost(a, b, eps, f, g, C=None, X=None, Y=None, long_double=False):
    """Transport cost <C,P> (Alg. 1, last step)."""
    return objectives(a, b, eps, f, g, C=C, X=X, Y=Y, long_double=long_double)["cost"]


def solve(a, b, eps, max_iter, tol=0.0, check_every=10, C=None, X=None, Y=None, f0=None, g0=None,
          err_every_iter=False, want_err=False, want_dual=False, long_double=False):
    """Alg. 1.  Returns dict(f, g, iters, converged, err_hist, dual_hist).

    ``tol <= 0`` runs exactly ``max_iter`` iterations.  ``err_hist[k-1]`` is the
    marginal error after iteration k (NaN where it was not evaluated);
    ``dual_hist[2(k-1)], dual_hist[2(k-1)+1]`` are D after the f and g half-steps."""
    head, n, m = _head(C, X, Y, a, b, eps)
    dt = _rdt(long_double)
    warm = f0 is not None or g0 is not None
    f = np.zeros(n, dtype=dt) if f0 is None else np.array(f0, dtype=dt)
    g = np.zeros(m, dtype=dt) if g0 is None else np.array(g0, dtype=dt)
    eh = np.full(max(max_iter, 1), np.nan, dtype=dt) if (want_err or err_every_iter) else None
    dh = np.full(2 * max(max_iter, 1), np.nan, dtype=dt) if want_dual else None
    conv = ctypes.c_int(0)
    it = _lib(long_double).fso_solve(*head, ctypes.c_int(int(max_iter)), ctypes.c_double(float(tol)),
                                     ctypes.c_int(int(check_every)), ctypes.c_int(int(warm)),
                                     ctypes.c_int(int(bool(err_every_iter))), _rp(f), _rp(g), _rp(eh), _rp(dh),
                                     ctypes.byref(conv))
    return dict(f=f, g=g, iters=int(it), converged=bool(conv.value),
                err_hist=None if eh is None else eh[:max_iter],
                dual_hist=None if dh is None else dh[:2 * max_iter])
