#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ for the five benchmark configurations.

Calls only the CPU oracle (oracle/) and the seeded input generators; nothing here touches the HIP
path.  Each .npz holds the oracle's fp64 potentials after the stated number of iterations, the
transport cost, the marginal error and the iteration count, for the exact fp32 inputs that
`paper_2605_00837_amd.workloads` regenerates from the seed.

    python tests/golden/make_golden.py c1 c2 c3 c4 c5 c5dense [--threads N] [--c4-iters K]
    python tests/golden/make_golden.py marginals      # adds the oracle's marginals to every stored file that lacks them

Every file also holds the oracle's row and column marginals of the plan of Eq. 5 at the stored
potentials (Sec. 4.5, each by its own LSE pass), which is what the plan-marginal bar compares with.
"""
import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2605_00837_amd import workloads as W  # noqa: E402


def _save(name, w, eps, r, extra=None):
    f, g = r["f"], r["g"]
    geo = dict(C=w.C, X=w.X, Y=w.Y)
    obj = oracle.objectives(w.a, w.b, eps, f, g, **geo)
    err = float(oracle.marginal_err(w.a, w.b, eps, f, g, **geo))
    rm, cm = oracle.marginals(w.a, w.b, eps, f, g, **geo)
    out = dict(f=f, g=g, iters=np.int64(r["iters"]), converged=np.int64(r["converged"]), eps=np.float64(eps),
               cost=np.float64(obj["cost"]), dual=np.float64(obj["dual"]), err=np.float64(err),
               n=np.int64(w.n), m=np.int64(w.m), row_marginal=rm, col_marginal=cm)
    if extra:
        out.update(extra)
    path = os.path.join(HERE, name + ".npz")
    np.savez_compressed(path, **out)
    print(f"wrote {path}: iters={r['iters']} converged={r['converged']} cost={obj['cost']:.9g} err={err:.3e}", flush=True)


def c1():
    w = W.c1_small_dense()
    _save("c1_dense256_200it", w, w.eps, oracle.solve(w.a, w.b, w.eps, 200, C=w.C))


def c2():
    w = W.c2_dense_gauss()
    # the configuration itself: tol = 1e-6, max 1000 iterations, checked every 10
    t = time.time()
    r = oracle.solve(w.a, w.b, w.eps, w.max_iter, tol=w.tol, check_every=10, C=w.C, want_err=True)
    eh = r["err_hist"]
    print(f"c2: {time.time() - t:.0f} s", flush=True)
    _save("c2_dense8192", w, w.eps, r, dict(err_hist=eh))
    # and a short fixed run, for a fast parity case at full size
    _save("c2_dense8192_50it", w, w.eps, oracle.solve(w.a, w.b, w.eps, 50, C=w.C))


def c3():
    w = W.c3_small_eps()
    for eps in w.eps_list:
        t = time.time()
        r = oracle.solve(w.a, w.b, eps, 2000, C=w.C)
        print(f"c3 eps={eps:g}: {time.time() - t:.0f} s", flush=True)
        _save(f"c3_dense4096_eps{eps:.0e}_2000it", w, eps, r)


def c4(iters):
    w = W.c4_sphere_points()
    t = time.time()
    r = oracle.solve(w.a, w.b, w.eps, iters, X=w.X, Y=w.Y)
    print(f"c4 {iters} it: {time.time() - t:.0f} s", flush=True)
    _save(f"c4_points65536_{iters}it", w, w.eps, r)


def c5():
    for m in (16384, 12288):
        w = W.c5_colour(16384, m)
        t = time.time()
        r = oracle.solve(w.a, w.b, w.eps, w.max_iter, tol=w.tol, check_every=10, X=w.X, Y=w.Y, want_err=True)
        print(f"c5 m={m}: {time.time() - t:.0f} s", flush=True)
        _save(f"c5_points16384x{m}", w, w.eps, r, dict(err_hist=r["err_hist"]))


def c5dense():
    """The dense variant of c5: the oracle is fed the fp32 matrix the dense kernels read."""
    for m in (16384, 12288):
        w = W.c5_colour(16384, m, dense=True)
        w.X = w.Y = None
        t = time.time()
        r = oracle.solve(w.a, w.b, w.eps, w.max_iter, tol=w.tol, check_every=10, C=w.C, want_err=True)
        print(f"c5 dense m={m}: {time.time() - t:.0f} s", flush=True)
        _save(f"c5_dense16384x{m}", w, w.eps, r, dict(err_hist=r["err_hist"]))


def _workload_of(name):
    """The inputs a stored file was made from, and its eps."""
    if name.startswith("c1_"):
        w = W.c1_small_dense(); return w, w.eps
    if name.startswith("c2_"):
        w = W.c2_dense_gauss(); return w, w.eps
    if name.startswith("c3_"):
        w = W.c3_small_eps()
        eps = [e for e in w.eps_list if f"eps{e:.0e}_" in name][0]
        return w, eps
    if name.startswith("c4_"):
        w = W.c4_sphere_points(); return w, w.eps
    if name.startswith("c5_"):
        m = int(name.split("x")[1])
        w = W.c5_colour(16384, m, dense="dense" in name)
        if "dense" in name:
            w.X = w.Y = None
        return w, w.eps
    raise ValueError(name)


def add_marginals():
    """Adds row_marginal / col_marginal (the oracle's, at the stored potentials) to files made before they were stored."""
    for fn in sorted(os.listdir(HERE)):
        if not fn.endswith(".npz"):
            continue
        path = os.path.join(HERE, fn)
        rec = dict(np.load(path))
        if "row_marginal" in rec:
            continue
        w, eps = _workload_of(fn[:-4])
        assert abs(float(rec["eps"]) - eps) < 1e-12 and int(rec["n"]) == w.n and int(rec["m"]) == w.m
        t = time.time()
        rm, cm = oracle.marginals(w.a, w.b, eps, rec["f"], rec["g"], C=w.C, X=w.X, Y=w.Y)
        # the stored error is the row-marginal error of the same potentials: the new arrays must reproduce it
        err = float(np.abs(rm - w.a.astype(np.float64)).sum())
        assert abs(err - float(rec["err"])) <= 1e-9 * max(1.0, float(rec["err"])) + 1e-13, (err, float(rec["err"]))
        rec.update(row_marginal=rm, col_marginal=cm)
        np.savez_compressed(path, **rec)
        print(f"{fn}: marginals added ({time.time() - t:.0f} s), row err {err:.3e}", flush=True)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("which", nargs="+")
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--c4-iters", type=int, default=500)
    a = ap.parse_args()
    if a.threads:
        oracle.set_threads(a.threads)
    for name in a.which:
        {"c1": c1, "c2": c2, "c3": c3, "c4": lambda: c4(a.c4_iters), "c5": c5, "c5dense": c5dense,
         "marginals": add_marginals}[name]()
