"""Pins for the CPU oracle: every check below compares the oracle with something
that is fixed by the paper's equations or by mathematics, not by the oracle
itself.  They are chosen so that a dropped log-weight, a wrong sign, a swapped
index or a Jacobi-instead-of-Gauss-Seidel update fails at least one of them.

The paper's own printed numbers (Tables 1-3: times, iteration counts, costs)
cannot serve as pins: their inputs are unseeded random histograms and the
tolerance is never stated.
"""
import itertools
import math

import numpy as np
import pytest
from scipy.special import logsumexp

from paper_2605_00837_amd import workloads as W

pytestmark = pytest.mark.filterwarnings("ignore::RuntimeWarning")


def _solve_converged(oracle, w, eps, iters=20000, tol=1e-13, **kw):
    return oracle.solve(w.a, w.b, eps, iters, tol=tol, check_every=10, C=w.C, X=w.X, Y=w.Y, **kw)


# ---- P1: brute-force exact OT over all permutations (Eq. 1; eps -> 0 limit, Sec. 3.2) ----
@pytest.mark.parametrize("n,seed", [(4, 0), (6, 1), (8, 2)])
def test_bruteforce_permutation_ot(oracle, n, seed):
    w = W.random_dense(n, n, seed=100 + seed, uniform=True)
    C = w.C.astype(np.float64)
    best = min(sum(C[i, s[i]] for i in range(n)) for s in itertools.permutations(range(n))) / n
    nt = oracle.max_threads()
    prev_gap = None
    oracle.set_threads(1)            # tiny problem, very many iterations: no thread fan-out
    try:
        for eps in (1e-1, 1e-2, 2e-3):
            r = _solve_converged(oracle, w, eps, iters=300000, tol=1e-11)
            err = float(oracle.marginal_err(w.a, w.b, eps, r["f"], r["g"], C=w.C))
            assert err < 1e-4
            cost = float(oracle.cost(w.a, w.b, eps, r["f"], r["g"], C=w.C))
            gap = cost - best
            # The plan's columns are exact and its rows are off by err in L1, so its cost is within
            # err * max C of a feasible plan's.  A feasible plan cannot beat the LP optimum, and
            # entropic optimality bounds the excess by eps * KL(sigma/n | a x b) = eps * ln n.
            slack = err * float(C.max()) + 1e-9
            assert gap >= -slack
            assert gap <= eps * math.log(n) + slack
            if prev_gap is not None:
                assert gap <= prev_gap + slack
            prev_gap = gap
    finally:
        oracle.set_threads(nt)
    assert abs(prev_gap) < 1e-4                         # eps -> 0 recovers the LP value


# ---- P2: huge eps gives the independent coupling a (x) b ----
def test_huge_eps_independent_coupling(oracle):
    w = W.random_dense(17, 23, seed=7)
    eps = 1e6
    r = oracle.solve(w.a, w.b, eps, 50, C=w.C)
    P = oracle.plan(w.a, w.b, eps, r["f"], r["g"], C=w.C)
    ab = np.outer(w.a.astype(np.float64), w.b.astype(np.float64))
    assert np.abs(P - ab).sum() < 5e-6
    # first-order form of the potential: f_i -> sum_j b_j C_ij + const
    lin = w.C.astype(np.float64) @ w.b.astype(np.float64)
    dev = (r["f"] - lin)
    assert np.ptp(dev) < 1e-5


# ---- P3: marginals. After a g-update columns are exact; after an f-update rows are exact;
#          the row error of Alg. 1 goes to zero. ----
def test_marginal_invariants(oracle):
    w = W.random_dense(40, 31, seed=11, eps=0.05)
    a64, b64 = w.a.astype(np.float64), w.b.astype(np.float64)
    r = oracle.solve(w.a, w.b, w.eps, 7, C=w.C)
    rr, cc = oracle.marginals(w.a, w.b, w.eps, r["f"], r["g"], C=w.C)
    assert np.abs(cc - b64).max() < 1e-13
    assert np.abs(rr - a64).sum() > 1e-8          # not yet converged: the row check is informative
    f2 = oracle.update_f(w.a, w.b, w.eps, r["g"], C=w.C)
    rr2, _ = oracle.marginals(w.a, w.b, w.eps, f2, r["g"], C=w.C)
    assert np.abs(rr2 - a64).max() < 1e-13
    # marginals agree with explicit sums over the explicit plan
    P = oracle.plan(w.a, w.b, w.eps, r["f"], r["g"], C=w.C)
    assert np.allclose(P.sum(1), rr, rtol=1e-12, atol=1e-15)
    assert np.allclose(P.sum(0), cc, rtol=1e-12, atol=1e-15)
    assert abs(oracle.marginal_err(w.a, w.b, w.eps, r["f"], r["g"], C=w.C) - np.abs(P.sum(1) - a64).sum()) < 1e-13
    long = oracle.solve(w.a, w.b, w.eps, 3000, C=w.C, err_every_iter=True)
    e = long["err_hist"]
    # fp32-normalised weights have sum a != sum b by a few 1e-9; at the fixed point r = a * sum b / sum a,
    # so the error floor is exactly |sum a - sum b|
    assert abs(e[-1] - abs(a64.sum() - b64.sum())) < 1e-13
    assert np.all(e[1:200] <= e[:199] * (1 + 1e-9) + 1e-15)     # decreasing on the way down


# ---- P4: dual objective is non-decreasing over every half-step; strong duality at convergence ----
@pytest.mark.parametrize("kind", ["dense", "points"])
def test_dual_monotone_and_strong_duality(oracle, kind):
    # weights exact in fp32 with sum exactly 1 on both sides: the marginal constraints are consistent
    w = (W.random_dense(30, 45, seed=5, eps=0.02, exact_weights=True) if kind == "dense"
         else W.random_points(33, 28, 3, seed=5, eps=0.02, exact_weights=True))
    r = oracle.solve(w.a, w.b, w.eps, 400, C=w.C, X=w.X, Y=w.Y, want_dual=True)
    D = r["dual_hist"]
    assert np.all(np.diff(D) >= -1e-12 * np.abs(D[1:]).max())
    assert D[3] - D[0] > 1e-6                                    # and it does move
    full = _solve_converged(oracle, w, w.eps)
    o = oracle.objectives(w.a, w.b, w.eps, full["f"], full["g"], C=w.C, X=w.X, Y=w.Y)
    assert abs(o["primal"] - o["dual"]) < 1e-11 * max(1.0, abs(o["primal"]))
    assert abs(o["mass"] - 1.0) < 1e-12
    # with sum P = 1 the dual is <a,f> + <b,g>
    a64, b64 = w.a.astype(np.float64), w.b.astype(np.float64)
    assert a64.sum() == 1.0 and b64.sum() == 1.0
    assert abs(o["dual"] - (a64 @ full["f"] + b64 @ full["g"])) < 1e-12
    assert o["kl"] > 0


# ---- P5: gauge invariance ----
def test_gauge_invariance(oracle):
    w = W.random_dense(21, 34, seed=3, eps=0.03)
    r = oracle.solve(w.a, w.b, w.eps, 25, C=w.C)
    c = 0.37
    P0 = oracle.plan(w.a, w.b, w.eps, r["f"], r["g"], C=w.C)
    P1 = oracle.plan(w.a, w.b, w.eps, r["f"] + c, r["g"] - c, C=w.C)
    assert np.allclose(P0, P1, rtol=1e-11, atol=0)
    assert abs(oracle.cost(w.a, w.b, w.eps, r["f"], r["g"], C=w.C)
               - oracle.cost(w.a, w.b, w.eps, r["f"] + c, r["g"] - c, C=w.C)) < 1e-12
    g_shift = oracle.update_g(w.a, w.b, w.eps, r["f"] + c, C=w.C)
    g_ref = oracle.update_g(w.a, w.b, w.eps, r["f"], C=w.C)
    assert np.abs(g_shift - (g_ref - c)).max() < 1e-13


# ---- P6: separable cost C_ij = u_i + v_j has a closed form after ONE iteration ----
def test_separable_cost_closed_form(oracle):
    rng = np.random.default_rng(42)
    n, m, eps = 19, 27, float(np.float32(0.07))
    u = rng.random(n).astype(np.float32)
    v = rng.random(m).astype(np.float32)
    C = (u[:, None].astype(np.float64) + v[None, :].astype(np.float64)).astype(np.float32)
    C64 = C.astype(np.float64)
    # the fp32-rounded matrix is what both sides see; make it exactly separable again
    u64 = C64[:, 0] - C64[0, 0]
    v64 = C64[0, :]
    if not np.array_equal(u64[:, None] + v64[None, :], C64):
        # choose dyadic values so that the fp32 sum is exact
        u = (rng.integers(0, 256, n) / 256.0).astype(np.float32)
        v = (rng.integers(0, 256, m) / 256.0).astype(np.float32)
        C = (u[:, None] + v[None, :]).astype(np.float32)
        u64, v64 = u.astype(np.float64), v.astype(np.float64)
    w = W.random_dense(n, m, seed=9)
    a64, b64 = w.a.astype(np.float64), w.b.astype(np.float64)
    r1 = oracle.solve(w.a, w.b, eps, 1, C=C, err_every_iter=True)
    kappa = -eps * np.log(np.sum(b64 * np.exp(-v64 / eps)))
    sa = a64.sum()
    assert np.abs(r1["f"] - (u64 + kappa)).max() < 1e-13
    assert np.abs(r1["g"] - (v64 - kappa - eps * np.log(sa))).max() < 1e-13
    P = oracle.plan(w.a, w.b, eps, r1["f"], r1["g"], C=C)
    assert np.abs(P - np.outer(a64, b64) / sa).max() < 1e-15
    assert r1["err_hist"][0] < 2e-7                  # |sum b / 1 - 1| from fp32-normalised weights only
    r5 = oracle.solve(w.a, w.b, eps, 5, C=C)
    # a fixed point up to the (sum a, sum b) normalisation constants, which only move the gauge
    P5 = oracle.plan(w.a, w.b, eps, r5["f"], r5["g"], C=C)
    assert np.abs(P5 - P).max() < 1e-9
    cost = oracle.cost(w.a, w.b, eps, r1["f"], r1["g"], C=C)
    assert abs(cost - (a64 @ u64 * b64.sum() + b64 @ v64 * a64.sum()) / sa) < 1e-13


# ---- P7: 2x2 closed form ----
def test_two_by_two_closed_form(oracle):
    C = np.array([[0.1, 0.9], [0.7, 0.2]], dtype=np.float32)
    a = np.array([0.5, 0.5], dtype=np.float32)
    eps = float(np.float32(0.25))
    r = oracle.solve(a, a, eps, 5000, tol=1e-15, check_every=1, C=C)
    P = oracle.plan(a, a, eps, r["f"], r["g"], C=C)
    C64 = C.astype(np.float64)
    s = math.exp(-(C64[0, 0] + C64[1, 1] - C64[0, 1] - C64[1, 0]) / (2 * eps))
    # P = [[t, .5-t],[.5-t, t]] with t/(.5-t) = exp(-(C11+C22-C12-C21)/(2 eps))
    t = 0.5 * s / (1 + s)
    assert abs(P[0, 0] - t) < 1e-13 and abs(P[1, 1] - t) < 1e-13
    assert abs(P[0, 1] - (0.5 - t)) < 1e-13 and abs(P[1, 0] - (0.5 - t)) < 1e-13


# ---- P8: one half-step equals SciPy's weighted logsumexp (independent LSE primitive) ----
@pytest.mark.parametrize("kind", ["dense", "points"])
def test_half_steps_match_scipy_logsumexp(oracle, kind):
    if kind == "dense":
        w = W.random_dense(37, 53, seed=21, eps=0.01, cmax=3.0)
        C64 = w.C.astype(np.float64)
    else:
        w = W.random_points(41, 29, 5, seed=22, eps=0.01)
        X64, Y64 = w.X.astype(np.float64), w.Y.astype(np.float64)
        C64 = ((X64[:, None, :] - Y64[None, :, :]) ** 2).sum(-1)
    rng = np.random.default_rng(1)
    g = rng.standard_normal(w.m)
    a64, b64 = w.a.astype(np.float64), w.b.astype(np.float64)
    f = oracle.update_f(w.a, w.b, w.eps, g, C=w.C, X=w.X, Y=w.Y)
    f_ref = -w.eps * logsumexp((g[None, :] - C64) / w.eps, b=b64[None, :], axis=1)
    assert np.abs(f - f_ref).max() < 1e-12
    g2 = oracle.update_g(w.a, w.b, w.eps, f, C=w.C, X=w.X, Y=w.Y)
    g_ref = -w.eps * logsumexp((f[:, None] - C64) / w.eps, b=a64[:, None], axis=0)
    assert np.abs(g2 - g_ref).max() < 1e-12
    # the solver's first iteration is exactly these two half-steps from zero, in Gauss-Seidel order
    r = oracle.solve(w.a, w.b, w.eps, 1, C=w.C, X=w.X, Y=w.Y)
    f1 = -w.eps * logsumexp((0 - C64) / w.eps, b=b64[None, :], axis=1)
    g1 = -w.eps * logsumexp((f1[:, None] - C64) / w.eps, b=a64[:, None], axis=0)
    assert np.abs(r["f"] - f1).max() < 1e-12 and np.abs(r["g"] - g1).max() < 1e-12
    g1_jacobi = -w.eps * logsumexp((0 - C64) / w.eps, b=a64[:, None], axis=0)
    assert np.abs(r["g"] - g1_jacobi).max() > 1e-3                # would catch a Jacobi-style update


# ---- P9: equivariance under permutation and transposition ----
def test_permutation_and_transpose_equivariance(oracle):
    w = W.random_dense(26, 31, seed=33, eps=0.04)
    r = oracle.solve(w.a, w.b, w.eps, 30, C=w.C)
    perm = np.random.default_rng(2).permutation(w.n)
    rp = oracle.solve(np.ascontiguousarray(w.a[perm]), w.b, w.eps, 30, C=np.ascontiguousarray(w.C[perm]))
    assert np.abs(rp["f"] - r["f"][perm]).max() < 1e-12
    assert np.abs(rp["g"] - r["g"]).max() < 1e-12
    Ct = np.ascontiguousarray(w.C.T)
    g = np.random.default_rng(3).standard_normal(w.m)
    f = oracle.update_f(w.a, w.b, w.eps, g, C=w.C)
    f_t = oracle.update_g(w.b, w.a, w.eps, g, C=Ct)     # transposed problem, roles swapped
    assert np.abs(f - f_t).max() < 1e-13


# ---- P10: double precision is itself converged (long-double rerun), incl. eps = 1e-4 ----
@pytest.mark.parametrize("eps", [1e-2, 1e-4])
def test_long_double_agreement(oracle, eps):
    w = W.c3_small_eps(48, 48)
    eps = float(np.float32(eps))
    r = oracle.solve(w.a, w.b, eps, 300, C=w.C)
    rl = oracle.solve(w.a, w.b, eps, 300, C=w.C, long_double=True)
    assert np.abs(r["f"] - rl["f"].astype(np.float64)).max() / eps < 1e-9
    assert np.abs(r["g"] - rl["g"].astype(np.float64)).max() / eps < 1e-9
    assert np.all(np.isfinite(r["f"])) and np.all(np.isfinite(r["g"]))


# ---- points path of the oracle equals the dense path on the exactly-evaluated cost ----
def test_points_equals_dense_on_same_cost(oracle):
    w = W.random_points(24, 37, 3, seed=8, eps=0.05)
    X64, Y64 = w.X.astype(np.float64), w.Y.astype(np.float64)
    C64 = ((X64[:, None, :] - Y64[None, :, :]) ** 2).sum(-1)
    rp = oracle.solve(w.a, w.b, w.eps, 40, X=w.X, Y=w.Y)
    a64, b64 = w.a.astype(np.float64), w.b.astype(np.float64)
    f, g = np.zeros(w.n), np.zeros(w.m)
    for _ in range(40):
        f = -w.eps * logsumexp((g[None, :] - C64) / w.eps, b=b64[None, :], axis=1)
        g = -w.eps * logsumexp((f[:, None] - C64) / w.eps, b=a64[:, None], axis=0)
    assert np.abs(rp["f"] - f).max() < 1e-11 and np.abs(rp["g"] - g).max() < 1e-11


# ---- zero weights: log = -inf, the entry carries no mass and its potential is unused ----
def test_zero_weight_entries(oracle):
    w = W.random_dense(12, 15, seed=4, eps=0.05)
    a = w.a.copy(); a[3] = 0.0; a /= a.sum(dtype=np.float64); a = a.astype(np.float32)
    b = w.b.copy(); b[5] = 0.0
    r = oracle.solve(a, b, w.eps, 200, C=w.C)
    assert np.all(np.isfinite(r["f"])) and np.all(np.isfinite(r["g"]))
    P = oracle.plan(a, b, w.eps, r["f"], r["g"], C=w.C)
    assert np.all(P[3] == 0) and np.all(P[:, 5] == 0)
    keep_r = np.arange(w.n) != 3
    keep_c = np.arange(w.m) != 5
    rs = oracle.solve(np.ascontiguousarray(a[keep_r]), np.ascontiguousarray(b[keep_c]), w.eps, 200,
                      C=np.ascontiguousarray(w.C[keep_r][:, keep_c]))
    assert np.abs(rs["f"] - r["f"][keep_r]).max() < 1e-12
    assert np.abs(rs["g"] - r["g"][keep_c]).max() < 1e-12


# ---- stopping rule of Alg. 1: checked only when k mod c == 0, first k with err < tol ----
def test_stopping_rule(oracle):
    w = W.random_dense(20, 20, seed=6, eps=0.05)
    full = oracle.solve(w.a, w.b, w.eps, 400, C=w.C, err_every_iter=True)
    e = full["err_hist"]
    tol = 1e-7
    for c in (1, 7, 10):
        r = oracle.solve(w.a, w.b, w.eps, 400, tol=tol, check_every=c, C=w.C)
        ks = [k for k in range(c, 401, c) if e[k - 1] < tol]
        assert r["converged"] and r["iters"] == ks[0]
    r = oracle.solve(w.a, w.b, w.eps, 5, tol=1e-30, check_every=1, C=w.C)
    assert (not r["converged"]) and r["iters"] == 5
    # warm start: k1 iterations then k2 more equals k1 + k2 in one go
    r1 = oracle.solve(w.a, w.b, w.eps, 13, C=w.C)
    r2 = oracle.solve(w.a, w.b, w.eps, 9, C=w.C, f0=r1["f"], g0=r1["g"])
    r3 = oracle.solve(w.a, w.b, w.eps, 22, C=w.C)
    assert np.array_equal(r2["f"], r3["f"]) and np.array_equal(r2["g"], r3["g"])


# ---- results do not depend on the OpenMP thread count ----
def test_thread_count_independence(oracle):
    w = W.random_dense(64, 50, seed=12, eps=0.02)
    nt = oracle.max_threads()
    try:
        oracle.set_threads(1)
        r1 = oracle.solve(w.a, w.b, w.eps, 20, C=w.C)
        oracle.set_threads(max(2, nt))
        r2 = oracle.solve(w.a, w.b, w.eps, 20, C=w.C)
    finally:
        oracle.set_threads(nt)
    assert np.array_equal(r1["f"], r2["f"]) and np.array_equal(r1["g"], r2["g"])


# ---- barycentric mapping (Sec. 5.6): pinned by what the projection must do in the cases where the
# ---- plan is known, not by re-typing its formula
def test_barycentric_projection_pins(oracle):
    rng = np.random.default_rng(12)
    # (a) huge eps: the plan is a (x) b, every row is mapped to the b-weighted mean of Z
    w = W.random_dense(13, 19, seed=31)
    Z = rng.standard_normal((19, 3))
    r = oracle.solve(w.a, w.b, 1e6, 50, C=w.C)
    T = oracle.barycentric(w.a, w.b, 1e6, r["f"], r["g"], Z, C=w.C)
    mean = (w.b.astype(np.float64)[:, None] * Z).sum(0) / w.b.astype(np.float64).sum()
    assert np.abs(T - mean[None, :]).max() < 1e-5
    # (b) constant Z is reproduced exactly whatever the potentials
    Zc = np.tile(np.array([[0.25, -3.0]]), (19, 1))
    f = rng.standard_normal(13)
    g = rng.standard_normal(19)
    T = oracle.barycentric(w.a, w.b, 0.3, f, g, Zc, C=w.C)
    assert np.abs(T - Zc[:13]).max() < 1e-13
    # (c) eps -> 0 on a uniform n x n problem: the plan concentrates on the optimal permutation found by
    #     brute force, so row i is mapped to Z[sigma(i)]
    n = 6
    wq = W.random_dense(n, n, seed=105, uniform=True)
    C = wq.C.astype(np.float64)
    best = min(itertools.permutations(range(n)), key=lambda s: sum(C[i, s[i]] for i in range(n)))
    Zq = rng.standard_normal((n, 2))
    nt = oracle.max_threads()
    oracle.set_threads(1)
    try:
        rq = _solve_converged(oracle, wq, 1e-3, iters=300000, tol=1e-11)
    finally:
        oracle.set_threads(nt)
    Tq = oracle.barycentric(wq.a, wq.b, 1e-3, rq["f"], rq["g"], Zq, C=wq.C)
    assert np.abs(Tq - Zq[list(best)]).max() < 1e-3
    # (d) the explicit plan and a library matrix product say the same (zero-weight row -> 0)
    w2 = W.random_points(11, 9, 3, seed=5)
    w2.a[3] = 0.0
    r2 = oracle.solve(w2.a, w2.b, 0.05, 5, X=w2.X, Y=w2.Y)
    Z2 = rng.standard_normal((9, 4))
    P = oracle.plan(w2.a, w2.b, 0.05, r2["f"], r2["g"], X=w2.X, Y=w2.Y)
    T2 = oracle.barycentric(w2.a, w2.b, 0.05, r2["f"], r2["g"], Z2, X=w2.X, Y=w2.Y)
    den = P.sum(1)
    ref = np.where(den[:, None] > 0, (P @ Z2) / np.where(den > 0, den, 1.0)[:, None], 0.0)
    assert np.abs(T2 - ref).max() < 1e-13 and np.all(T2[3] == 0.0)
