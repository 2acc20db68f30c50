"""Time what runs around the iteration loop, on the GPU: plan, cost, one-pass diagnostics and barycentric
mapping at the headline size and at the point-cloud size; the single-workgroup kernel, the one-launch
multi-workgroup kernel (dense and point clouds) against the multi-kernel path, and batched solves.

    python -m paper_2605_00837_amd.report_extras
"""
from __future__ import annotations

import time


def main():
    import torch
    from . import binding as fs, workloads as W

    def timeit(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    print("| call | workload | us per call |")
    print("|---|---|---|")
    w = W.c2_dense_gauss()
    C, a, b = (torch.from_numpy(t).cuda() for t in (w.C, w.a, w.b))
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 100, 0.0, C=C, want_f64=True)
    f, g = r["f64"], r["g64"]
    P = torch.empty((w.n, w.m), dtype=torch.float32, device="cuda")
    Z = torch.randn((w.m, 3), device="cuda")
    tag = f"dense {w.n} x {w.m}"
    print(f"| fs_plan | {tag} | {timeit(lambda: fs.fs_plan(a, b, w.eps, f, g, C=C, P=P)):.1f} |", flush=True)
    print(f"| fs_cost | {tag} | {timeit(lambda: fs.fs_cost(a, b, w.eps, f, g, C=C)):.1f} |", flush=True)
    print(f"| fs_diagnostics | {tag} | {timeit(lambda: fs.fs_diagnostics(a, b, w.eps, f, g, C=C)):.1f} |", flush=True)
    print(f"| fs_barycentric (dz = 3) | {tag} | {timeit(lambda: fs.fs_barycentric(a, b, w.eps, f, g, Z, C=C)):.1f} |", flush=True)
    del C, P
    w = W.c4_sphere_points()
    X, Y, a, b = (torch.from_numpy(t).cuda() for t in (w.X, w.Y, w.a, w.b))
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 50, 0.0, X=X, Y=Y, want_f64=True)
    f, g = r["f64"], r["g64"]
    tag = f"points {w.n} x {w.m}, d = 3"
    print(f"| fs_cost | {tag} | {timeit(lambda: fs.fs_cost(a, b, w.eps, f, g, X=X, Y=Y), 3):.0f} |", flush=True)
    print(f"| fs_diagnostics | {tag} | {timeit(lambda: fs.fs_diagnostics(a, b, w.eps, f, g, X=X, Y=Y), 3):.0f} |", flush=True)
    print(f"| fs_barycentric (Z = Y) | {tag} | {timeit(lambda: fs.fs_barycentric(a, b, w.eps, f, g, Y, X=X, Y=Y), 3):.0f} |", flush=True)
    del X, Y
    for n in (512, 4096):
        w = W.random_points(n, n, 3, seed=1, eps=0.05)
        X, Y, a, b = (torch.from_numpy(t).cuda() for t in (w.X, w.Y, w.a, w.b))
        r = fs.fs_sinkhorn_solve(a, b, w.eps, 30, 0.0, X=X, Y=Y, want_f64=True)
        f, g = r["f64"], r["g64"]
        tag = f"points {n} x {n}, d = 3"
        print(f"| fs_cost | {tag} | {timeit(lambda: fs.fs_cost(a, b, w.eps, f, g, X=X, Y=Y), 100):.1f} |", flush=True)
        print(f"| fs_diagnostics | {tag} | {timeit(lambda: fs.fs_diagnostics(a, b, w.eps, f, g, X=X, Y=Y), 100):.1f} |", flush=True)
        print(f"| fs_barycentric (Z = Y) | {tag} | {timeit(lambda: fs.fs_barycentric(a, b, w.eps, f, g, Y, X=X, Y=Y), 100):.1f} |", flush=True)

    print()
    print("| solve | iterations | ms | per problem-iteration |")
    print("|---|---|---|---|")
    for n in (64, 128, 256):
        w = W.random_dense(n, n, seed=1, cmax=1.0, eps=0.05)
        C, a, b = (torch.from_numpy(t).cuda() for t in (w.C, w.a, w.b))
        for mode, name in ((3, "single-workgroup kernel"), (2, "multi-kernel path")):
            fs.fs_sinkhorn_solve(a, b, w.eps, 10, 0.0, C=C, kernel_mode=mode)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fs.fs_sinkhorn_solve(a, b, w.eps, 2000, 0.0, C=C, kernel_mode=mode)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            print(f"| {n} x {n}, {name} | 2000 | {dt * 1e3:.2f} | {dt / 2000 * 1e6:.2f} us |", flush=True)
    for n in (256, 384, 512, 1024, 2048):
        w = W.random_dense(n, n, seed=1, cmax=1.0, eps=0.05)
        C, a, b = (torch.from_numpy(t).cuda() for t in (w.C, w.a, w.b))
        for mode, name in ((4, "one launch, up to 32 workgroups"), (5, "one launch, whole chip"), (2, "multi-kernel path")):
            if mode == 4 and n > 1024:
                continue
            fs.fs_sinkhorn_solve(a, b, w.eps, 10, 0.0, C=C, kernel_mode=mode)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fs.fs_sinkhorn_solve(a, b, w.eps, 2000, 0.0, C=C, kernel_mode=mode)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            print(f"| {n} x {n}, {name} | 2000 | {dt * 1e3:.2f} | {dt / 2000 * 1e6:.2f} us |", flush=True)
    for n, d in ((200, 3), (512, 3), (200, 16), (1024, 3), (2048, 3)):
        w = W.random_points(n, n, d, seed=1, eps=0.05)
        X, Y, a, b = (torch.from_numpy(t).cuda() for t in (w.X, w.Y, w.a, w.b))
        for mode, name in ((0, "automatic"), (1, "multi-kernel path")):
            fs.fs_sinkhorn_solve(a, b, w.eps, 10, 0.0, X=X, Y=Y, kernel_mode=mode)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fs.fs_sinkhorn_solve(a, b, w.eps, 1000, 0.0, X=X, Y=Y, kernel_mode=mode)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            print(f"| points {n} x {n}, d = {d}, {name} | 1000 | {dt * 1e3:.2f} | {dt / 1000 * 1e6:.2f} us |", flush=True)
    for B, n in ((256, 64), (256, 128), (256, 256), (1024, 256)):
        Cb = torch.rand((B, n, n), device="cuda")
        ab = torch.full((B, n), 1.0 / n, device="cuda")
        fs.fs_sinkhorn_dense_batched(Cb, ab, ab, 0.05, 10, 0.0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fs.fs_sinkhorn_dense_batched(Cb, ab, ab, 0.05, 500, 0.0)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        print(f"| batch of {B}, {n} x {n} | 500 | {dt * 1e3:.2f} | {dt / 500 / B * 1e9:.1f} ns |", flush=True)


if __name__ == "__main__":
    main()
