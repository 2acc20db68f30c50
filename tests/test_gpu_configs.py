"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration
bench.py times (library defaults), against oracle results stored under tests/golden/ by
tests/golden/make_golden.py (which calls only the CPU oracle).

Spec bars: potentials max|df|/eps <= 1e-3 (fp32 outputs), plan-marginal L1 difference
<= 1e-5, transport-cost relative error <= 1e-4.  The fp64 outputs are held to 2e-5.
"""
import os

import numpy as np
import pytest

from paper_2605_00837_amd import workloads as W

pytestmark = pytest.mark.gpu

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TOL_F32, TOL_F64, TOL_MARG, TOL_COST = 1e-3, 2e-5, 1e-5, 1e-4


@pytest.fixture(scope="module")
def fs():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_00837_amd import binding
    return binding


def gold(name):
    path = os.path.join(GOLD, name + ".npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated (python tests/golden/make_golden.py)")
    return np.load(path)


def dev(x):
    import torch
    return None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()


def check(fs, oracle, w, eps, r, g, tol64=TOL_F64):
    """All three spec bars.  r: GPU result dict with f, g, f64, g64; g: stored oracle record."""
    f64, g64 = r["f64"].cpu().numpy(), r["g64"].cpu().numpy()
    f32, g32 = r["f"].cpu().numpy().astype(np.float64), r["g"].cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(f32)) and np.all(np.isfinite(g32)) and not r["nonfinite"]
    e32 = max(np.abs(f32 - g["f"]).max(), np.abs(g32 - g["g"]).max()) / eps
    assert e32 < TOL_F32, e32                     # the spec bar, on the raw fp32 potentials
    # The tighter bar on the fp64 outputs is taken after removing the shift (f + c, g - c), which leaves
    # the plan unchanged: nothing in the iteration damps that direction, so the rounding bias of the
    # fp32 sums (about 1e-8 eps per iteration) adds up along it over thousands of iterations.  The raw
    # figure is held to the spec bar as well and printed beside the corrected one.
    df, dg = f64 - g["f"], g64 - g["g"]
    raw64 = max(np.abs(df).max(), np.abs(dg).max()) / eps
    assert raw64 < TOL_F32, raw64
    c = 0.5 * (df.mean() - dg.mean())
    assert abs(c) / eps < TOL_F32, c / eps
    e64 = max(np.abs(df - c).max(), np.abs(dg + c).max()) / eps
    assert e64 < tol64, e64
    geo = dict(C=dev(w.C), X=dev(w.X), Y=dev(w.Y))
    a, b = dev(w.a), dev(w.b)
    cost = float(fs.fs_cost(a, b, eps, r["f"], r["g"], **geo).cpu()[0])
    assert abs(cost - float(g["cost"])) <= TOL_COST * abs(float(g["cost"])), (cost, float(g["cost"]))
    # Plan marginals (plan of Eq. 5, marginals of Sec. 4.5): the oracle's marginals at its own potentials
    # are stored; those of the GPU's potentials are rebuilt (a) by the oracle on the CPU and (b) by the
    # library's own one-pass diagnostics kernel, both from the fp64 potentials (an fp32 potential of
    # size 1 is only good to 6e-8 / eps in the exponent, i.e. 6e-5 of every plan entry at eps = 1e-3).
    ro, co = g["row_marginal"], g["col_marginal"]
    rg, cg = oracle.marginals(w.a, w.b, eps, f64, g64, C=w.C, X=w.X, Y=w.Y)
    l1_cpu = np.abs(rg - ro).sum() + np.abs(cg - co).sum()
    assert l1_cpu <= TOL_MARG, l1_cpu
    d = fs.fs_diagnostics(a, b, eps, r["f64"], r["g64"], want_marginals=True, **geo)
    rd, cd = d["row_marginal"].cpu().numpy(), d["col_marginal"].cpu().numpy()
    l1_gpu = np.abs(rd - ro).sum() + np.abs(cd - co).sum()
    assert l1_gpu <= TOL_MARG, l1_gpu
    print(f"  |dpot|/eps fp32 {e32:.2e}, fp64 raw {raw64:.2e}, fp64 without the shift {e64:.2e}; "
          f"marginal L1 {l1_cpu:.2e} (oracle pass), {l1_gpu:.2e} (diagnostics kernel); cost {cost:.9g}")
    return e64, e32


def test_c1_dense256(fs, oracle):
    g = gold("c1_dense256_200it")
    w = W.c1_small_dense()
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, 200, 0.0, C=dev(w.C), want_f64=True)
    assert r["iters"] == 200 == int(g["iters"])
    check(fs, oracle, w, w.eps, r, g)
    assert abs(r["marginal_err"] - float(g["err"])) < 5e-7


def test_c2_dense8192_headline(fs, oracle):
    w = W.c2_dense_gauss()
    a, b, C = dev(w.a), dev(w.b), dev(w.C)
    g50 = gold("c2_dense8192_50it")
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 50, 0.0, C=C, want_f64=True)
    check(fs, oracle, w, w.eps, r, g50)
    g = gold("c2_dense8192")
    # the configuration itself: stop at err < 1e-6 or 1000 iterations (it does not get there in 1000)
    r = fs.fs_sinkhorn_solve(a, b, w.eps, w.max_iter, w.tol, C=C, want_f64=True, check_every=10)
    assert r["iters"] == int(g["iters"]) and r["converged"] == bool(g["converged"])
    check(fs, oracle, w, w.eps, r, g)
    assert abs(r["marginal_err"] - float(g["err"])) <= 1e-3 * float(g["err"]) + 5e-7
    # the two spec entry points give the same potentials
    f2, g2, it2 = fs.fs_sinkhorn_dense(C, a, b, w.eps, w.max_iter, w.tol)
    assert it2 == r["iters"]
    assert float((f2 - r["f"]).abs().max()) / w.eps < 1e-5


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_c3_small_eps_sweep(fs, oracle, idx):
    w = W.c3_small_eps()
    eps = w.eps_list[idx]
    g = gold(f"c3_dense4096_eps{eps:.0e}_2000it")
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), eps, 2000, 0.0, C=dev(w.C), want_f64=True)
    assert r["iters"] == 2000
    check(fs, oracle, w, eps, r, g)


def test_c4_points_sphere(fs, oracle):
    cands = [n for n in os.listdir(GOLD) if n.startswith("c4_points65536_")]
    if not cands:
        pytest.skip("no c4 golden file")
    name = sorted(cands, key=lambda s: int(s.split("_")[2][:-6]))[-1][:-4]
    g = gold(name)
    iters = int(g["iters"])
    w = W.c4_sphere_points()
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, iters, 0.0, X=dev(w.X), Y=dev(w.Y), want_f64=True)
    assert r["iters"] == iters
    check(fs, oracle, w, w.eps, r, g)
    assert abs(r["marginal_err"] - float(g["err"])) <= 1e-3 * float(g["err"]) + 5e-7
    f2, g2, it2 = fs.fs_sinkhorn_points(dev(w.X), dev(w.Y), dev(w.a), dev(w.b), w.eps, 20, 0.0)
    assert it2 == 20 and bool(f2.isfinite().all())


@pytest.mark.parametrize("m", [16384, 12288])
def test_c5_colour_points_and_dense(fs, oracle, m):
    g = gold(f"c5_points16384x{m}")
    w = W.c5_colour(16384, m, dense=True)
    a, b, X, Y = dev(w.a), dev(w.b), dev(w.X), dev(w.Y)
    k_orc = int(g["iters"])
    # the configuration itself: run to err < 1e-5; the device check may fire one interval apart
    r = fs.fs_sinkhorn_solve(a, b, w.eps, w.max_iter, w.tol, X=X, Y=Y, check_every=10)
    assert r["converged"] == bool(g["converged"])
    assert abs(r["iters"] - k_orc) <= 10, (r["iters"], k_orc)
    # parity at the oracle's iteration count
    r = fs.fs_sinkhorn_solve(a, b, w.eps, k_orc, 0.0, X=X, Y=Y, want_f64=True)
    wp = W.c5_colour(16384, m)            # points only
    check(fs, oracle, wp, w.eps, r, g)
    # dense variant from the same points, against the oracle fed the same fp32 matrix (C is the fp32
    # rounding of the exact cost, so its potentials differ from the point-cloud ones at the 1e-4 level)
    gd = gold(f"c5_dense16384x{m}")
    kd = int(gd["iters"])
    C = dev(w.C)
    rd = fs.fs_sinkhorn_solve(a, b, w.eps, w.max_iter, w.tol, C=C, check_every=10)
    assert rd["converged"] == bool(gd["converged"])
    assert abs(rd["iters"] - kd) <= 10, (rd["iters"], kd)
    rd = fs.fs_sinkhorn_solve(a, b, w.eps, kd, 0.0, C=C, want_f64=True)
    wd = W.Workload(w.name, w.n, w.m, w.a, w.b, w.eps, w.max_iter, w.tol, C=w.C)
    check(fs, oracle, wd, w.eps, rd, gd)
