"""Seeded synthetic inputs for the log-domain Sinkhorn hot path.

This module only draws random numbers and assembles arrays; it contains none of
the method's arithmetic (no LogSumExp, no potentials).  It is the single source
of inputs for both the HIP path and the CPU oracle: each workload returns the
exact fp32 arrays handed to either side.

Recipe (all workloads): ``numpy.random.default_rng(seed)`` (PCG64), draws are
made in fp64 in the order written below, then rounded to fp32.  A dense cost
matrix is built in fp64 from the *fp32-rounded* points and then rounded to
fp32.  Seeds are ``83700 + k`` for workload ``k``.

The five workloads stand in for the paper's experiments, whose own inputs
(unseeded histograms on a 1-D grid, two photographs, a 200-point cloud) are not
available: sizes follow the paper's Table 1 / Table 3 (n = 256 ... 8192), the
stability sweep of Sec. 5.4, the point-cloud matching and colour transfer of
Sec. 5.6.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

SEED_BASE = 83700


@dataclass
class Workload:
    """One optimal-transport problem instance (all arrays fp32, C-contiguous)."""
    name: str
    n: int
    m: int
    a: np.ndarray                 # [n] source weights, sum ~ 1
    b: np.ndarray                 # [m] target weights, sum ~ 1
    eps: float                    # regularisation (the fp32 value, as a python float)
    max_iter: int
    tol: float                    # <= 0: run exactly max_iter iterations
    C: Optional[np.ndarray] = None   # [n, m] dense cost, or None
    X: Optional[np.ndarray] = None   # [n, d] points, or None
    Y: Optional[np.ndarray] = None   # [m, d]
    eps_list: Sequence[float] = field(default_factory=tuple)   # sweep values, if any

    @property
    def d(self) -> int:
        return 0 if self.X is None else int(self.X.shape[1])


def _f32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))


def _eps32(eps: float) -> float:
    """The regularisation as the fp32 value that crosses the C ABI."""
    return float(np.float32(eps))


def sqdist_f32(X32: np.ndarray, Y32: np.ndarray, chunk: int = 1024) -> np.ndarray:
    """||x_i - y_j||^2 in fp64 from fp32 points, rounded to fp32, built in row chunks."""
    n, m = X32.shape[0], Y32.shape[0]
    Y64 = Y32.astype(np.float64)
    C = np.empty((n, m), dtype=np.float32)
    for i0 in range(0, n, chunk):
        Xc = X32[i0:i0 + chunk].astype(np.float64)
        D = np.zeros((Xc.shape[0], m), dtype=np.float64)
        for t in range(X32.shape[1]):
            diff = Xc[:, t][:, None] - Y64[:, t][None, :]
            D += diff * diff
        C[i0:i0 + chunk] = D.astype(np.float32)
    return C


def _uniform_weights(k: int) -> np.ndarray:
    return np.full(k, np.float32(1.0 / k), dtype=np.float32)


def _dirichlet(rng, k: int, shape: float) -> np.ndarray:
    w = rng.gamma(shape, 1.0, size=k)
    return _f32(w / w.sum())


def _dyadic_weights(rng, k: int, bits: int = 20) -> np.ndarray:
    """Non-uniform positive weights that are exact in fp32 and sum to exactly 1:
    integer counts (each >= 1) that total 2**bits, divided by 2**bits."""
    total = 1 << bits
    p = rng.gamma(1.0, 1.0, size=k)
    counts = 1 + rng.multinomial(total - k, p / p.sum())
    return (counts.astype(np.float64) / total).astype(np.float32)


def c1_small_dense(n: int = 256, m: Optional[int] = None, seed: int = SEED_BASE + 1) -> Workload:
    """2-D uniform points, dense squared-Euclidean cost, uniform weights, eps=0.05, 200 iterations."""
    m = n if m is None else m
    rng = np.random.default_rng(seed)
    X = _f32(rng.random((n, 2)))
    Y = _f32(rng.random((m, 2)))
    return Workload("c1_dense_uniform2d", n, m, _uniform_weights(n), _uniform_weights(m),
                    _eps32(0.05), 200, 0.0, C=sqdist_f32(X, Y))


def c2_dense_gauss(n: int = 8192, m: Optional[int] = None, seed: int = SEED_BASE + 2) -> Workload:
    """X~N(0,I2), Y~N((1,1),0.5 I2), dense fp32 cost, Dirichlet(1) weights, eps=1e-2,
    stop at marginal error < 1e-6 or 1000 iterations (the headline configuration)."""
    m = n if m is None else m
    rng = np.random.default_rng(seed)
    X = _f32(rng.standard_normal((n, 2)))
    Y = _f32(1.0 + np.sqrt(0.5) * rng.standard_normal((m, 2)))
    a = _dirichlet(rng, n, 1.0)
    b = _dirichlet(rng, m, 1.0)
    return Workload("c2_dense_gauss2d", n, m, a, b, _eps32(1e-2), 1000, 1e-6, C=sqdist_f32(X, Y))


def c3_small_eps(n: int = 4096, m: Optional[int] = None, seed: int = SEED_BASE + 3) -> Workload:
    """2-D uniform points, cost normalised to max 1, uniform weights, eps sweep
    {1e-1,1e-2,1e-3,1e-4}, 2000 fixed iterations each."""
    m = n if m is None else m
    rng = np.random.default_rng(seed)
    X = _f32(rng.random((n, 2)))
    Y = _f32(rng.random((m, 2)))
    X64, Y64 = X.astype(np.float64), Y.astype(np.float64)
    D = np.zeros((n, m), dtype=np.float64)
    for t in range(2):
        diff = X64[:, t][:, None] - Y64[:, t][None, :]
        D += diff * diff
    D /= D.max()
    eps_list = tuple(_eps32(e) for e in (1e-1, 1e-2, 1e-3, 1e-4))
    return Workload("c3_small_eps_sweep", n, m, _uniform_weights(n), _uniform_weights(m),
                    eps_list[0], 2000, 0.0, C=np.ascontiguousarray(D.astype(np.float32)),
                    eps_list=eps_list)


def c4_sphere_points(n: int = 65536, seed: int = SEED_BASE + 4) -> Workload:
    """3-D noisy unit sphere, target = rotated + shifted copy, uniform weights,
    eps=1e-3, 500 fixed iterations, cost never materialised (n = m)."""
    rng = np.random.default_rng(seed)
    Z = rng.standard_normal((n, 3))
    Z /= np.linalg.norm(Z, axis=1, keepdims=True)
    X64 = Z + 0.1 * rng.standard_normal((n, 3))        # N(0, 0.01 I): sigma = 0.1
    Q, R = np.linalg.qr(rng.standard_normal((3, 3)))
    Q = Q * np.sign(np.diag(R))[None, :]
    if np.linalg.det(Q) < 0:
        Q[:, 0] = -Q[:, 0]
    Y64 = X64 @ Q.T + np.array([0.1, 0.0, 0.0])
    return Workload("c4_points_sphere3d", n, n, _uniform_weights(n), _uniform_weights(n),
                    _eps32(1e-3), 500, 0.0, X=_f32(X64), Y=_f32(Y64))


def _gmm_rgb(rng, k: int, comps: int = 8) -> np.ndarray:
    w = rng.gamma(1.0, 1.0, size=comps)
    w /= w.sum()
    means = rng.uniform(0.15, 0.85, size=(comps, 3))
    A = 0.08 * rng.standard_normal((comps, 3, 3))
    cov = A @ np.transpose(A, (0, 2, 1)) + 4e-4 * np.eye(3)[None]
    L = np.linalg.cholesky(cov)
    which = rng.choice(comps, size=k, p=w)
    z = rng.standard_normal((k, 3))
    pts = means[which] + np.einsum("kij,kj->ki", L[which], z)
    return np.clip(pts, 0.0, 1.0)


def c5_colour(n: int = 16384, m: Optional[int] = None, seed: int = SEED_BASE + 5,
              dense: bool = False) -> Workload:
    """RGB clouds from two 8-component Gaussian mixtures, Dirichlet(2) weights,
    eps=5e-3, run to marginal error < 1e-5 (cap 2000).  ``m=12288`` gives the
    rectangular variant; ``dense=True`` also materialises C from the same points."""
    m = n if m is None else m
    rng = np.random.default_rng(seed)
    X = _f32(_gmm_rgb(rng, n))
    Y = _f32(_gmm_rgb(rng, m))
    a = _dirichlet(rng, n, 2.0)
    b = _dirichlet(rng, m, 2.0)
    w = Workload("c5_colour_rgb", n, m, a, b, _eps32(5e-3), 2000, 1e-5, X=X, Y=Y)
    if dense:
        w.C = sqdist_f32(X, Y)
    return w


def random_dense(n: int, m: int, seed: int, cmax: float = 1.0, eps: float = 0.05,
                 uniform: bool = False, exact_weights: bool = False) -> Workload:
    """Generic test instance: i.i.d. U[0,cmax) costs (no geometry); Dirichlet(1), uniform, or
    (exact_weights) non-uniform dyadic weights whose fp32 values sum to exactly 1."""
    rng = np.random.default_rng(seed)
    C = _f32(cmax * rng.random((n, m)))
    if uniform:
        a, b = _uniform_weights(n), _uniform_weights(m)
    elif exact_weights:
        a, b = _dyadic_weights(rng, n), _dyadic_weights(rng, m)
    else:
        a, b = _dirichlet(rng, n, 1.0), _dirichlet(rng, m, 1.0)
    return Workload(f"random_dense_{n}x{m}", n, m, a, b, _eps32(eps), 100, 0.0, C=C)


def random_points(n: int, m: int, d: int, seed: int, eps: float = 0.05,
                  exact_weights: bool = False) -> Workload:
    """Generic point-cloud test instance: N(0, I_d)/sqrt(d) clouds, Dirichlet(1) (or dyadic) weights."""
    rng = np.random.default_rng(seed)
    X = _f32(rng.standard_normal((n, d)) / np.sqrt(d))
    Y = _f32(0.3 + rng.standard_normal((m, d)) / np.sqrt(d))
    wgt = _dyadic_weights if exact_weights else (lambda r, k: _dirichlet(r, k, 1.0))
    return Workload(f"random_points_{n}x{m}x{d}", n, m, wgt(rng, n), wgt(rng, m), _eps32(eps), 100, 0.0,
                    X=X, Y=Y)
