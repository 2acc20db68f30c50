"""Run the five benchmark configurations on the GPU and print a markdown table:
iterations, convergence, time to stop and time per iteration (median and minimum of `--reps` runs,
inputs resident on the device, one warm-up run before).

    python -m paper_2605_00837_amd.report_configs [--reps 5] [--only c1,c2,...]
"""
from __future__ import annotations

import argparse
import statistics
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--only", default="c1,c2,c2_fixed,c2_check1,c2_half,c3,c4,c5")
    args = ap.parse_args()
    import torch
    from . import binding as fs, workloads as W

    def dev(x):
        return None if x is None else torch.from_numpy(x).cuda()

    def timed(label, w, eps, max_iter, tol, dense=True, cost_dtype=None, **kw):
        geo = dict(C=dev(w.C)) if dense else dict(X=dev(w.X), Y=dev(w.Y))
        if cost_dtype is not None:                   # the same matrix stored in 2 bytes per entry
            geo["C"] = geo["C"].to(cost_dtype)
        a, b = dev(w.a), dev(w.b)
        fs.fs_sinkhorn_solve(a, b, eps, min(max_iter, 20), 0.0, **geo, **kw)
        torch.cuda.synchronize()
        ts, r = [], None
        for _ in range(args.reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            r = fs.fs_sinkhorn_solve(a, b, eps, max_iter, tol, **geo, **kw)
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        med, mn = statistics.median(ts), min(ts)
        print(f"| {label} | {r['iters']} | {'yes' if r['converged'] else 'no'} | {r['marginal_err']:.3e} | "
              f"{med * 1e3:.3f} | {mn * 1e3:.3f} | {med * 1e6 / max(r['iters'], 1):.2f} |", flush=True)

    only = set(args.only.split(","))
    print("| configuration | iterations | converged | err | ms to stop (median) | (min) | us / iteration |")
    print("|---|---|---|---|---|---|---|")
    if "c1" in only:
        w = W.c1_small_dense()
        timed("c1 dense 256x256 eps 0.05, 200 fixed", w, w.eps, 200, 0.0)
        timed("c1, single-workgroup kernel", w, w.eps, 200, 0.0, kernel_mode=3)
    if only & {"c2", "c2_fixed", "c2_check1", "c2_half"}:
        w = W.c2_dense_gauss()
        if "c2" in only:
            timed("c2 dense 8192x8192 eps 1e-2, tol 1e-6, check every 10", w, w.eps, w.max_iter, w.tol, check_every=10)
        if "c2_check1" in only:
            timed("c2, check every iteration", w, w.eps, w.max_iter, w.tol, check_every=1)
        if "c2_fixed" in only:
            timed("c2, 1000 fixed iterations", w, w.eps, 1000, 0.0)
        if "c2_half" in only:
            timed("c2 with C stored as fp16, 1000 fixed iterations", w, w.eps, 1000, 0.0, cost_dtype=torch.float16)
            timed("c2 with C stored as bfloat16, 1000 fixed iterations", w, w.eps, 1000, 0.0, cost_dtype=torch.bfloat16)
    if "c3" in only:
        w = W.c3_small_eps()
        for eps in w.eps_list:
            timed(f"c3 dense 4096x4096 eps {eps:g}, 2000 fixed", w, eps, 2000, 0.0)
    if "c4" in only:
        w = W.c4_sphere_points()
        timed("c4 points 65536 x 65536 d=3 eps 1e-3, 500 fixed", w, w.eps, 500, 0.0, dense=False)
    if "c5" in only:
        for m in (16384, 12288):
            w = W.c5_colour(16384, m, dense=True)
            timed(f"c5 points 16384 x {m} eps 5e-3, tol 1e-5", w, w.eps, w.max_iter, w.tol, dense=False, check_every=10)
            timed(f"c5 dense (same points, C stored)", w, w.eps, w.max_iter, w.tol, check_every=10)


if __name__ == "__main__":
    main()
