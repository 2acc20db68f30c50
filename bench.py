#!/usr/bin/env python3
"""Benchmark of the log-domain Sinkhorn hot path on one MI355X; one JSON line per run.

A "step" is one pass of the whole hot path -- f-update (row LSE), g-update (column LSE with the new f) and the
marginal-error check -- over one of the five seeded synthetic workloads (`--workload`, default c2: the dense
n = m = 8192 fp32 problem at eps = 1e-2 that the headline metric is quoted on).  Inputs are resident in HBM
before the timed region starts; the timed region is one blocking solve of K iterations between synchronisations.

    python bench.py [--workload c1|c2|c3|c4|c5p|c5d] [--steps K] [--warmup W]
    python bench.py --calibrate-read      # the read rate a plain streaming kernel reaches (practical ceiling beside the peak)
    python bench.py --calibrate-copy      # a plain 256 MiB device copy: what the FETCH_SIZE / WRITE_SIZE counters
                                          # read for a known size (run under rocprofv3 --pmc)

Every line carries `roofline` (the dominant kernel: algorithmic bytes or operations per launch over its average
launch duration, measured in the run with events that the runtime stamps with the start and the stop of the
dispatch), for the dense workloads `iteration` (the whole iteration against the same HBM peak: algorithmic bytes
of one iteration over the wall-clock time per step) and `cpu_baseline` (the CPU oracle as it stands on a bounded
sample of the same workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP64_VECTOR_PEAK_TFLOPS = 78.6
# v_exp_f32 takes 8 issue cycles per wave64 instruction (half the rate of a plain fp32 or fp64 instruction):
# 256 compute units x 4 SIMDs x 64 lanes x 2.4 GHz / 8.  The point-cloud kernel's measured time fits this
# figure together with 4 cycles for each of its other instructions to within 1 %.
EXP_PEAK_PER_S = 256 * 4 * 64 * 2.4e9 / 8


def _traffic_from_profiles(kernel, n, m):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of the same
    workload (counters are collected in runs of their own, not in this run)."""
    for name in ("k_resident_c2_dense8192_pmc.json", "k_persist_c2_dense8192_pmc.json"):
        path = os.path.join(ROOT, "profiles", name)
        try:
            with open(path) as fh:
                rec = json.load(fh)
            if rec.get("n") == n and rec.get("m") == m and rec.get("kernel", "").startswith(kernel):
                return rec.get("hbm_bytes_per_launch"), os.path.relpath(path, ROOT)
        except (OSError, ValueError):
            pass
    return None, None


def _oracle_rate(solve, budget_s, unit_per_iter, max_iters=200):
    """Times `solve(iters)` (the oracle, Alg. 1 with the paper's check interval) for about budget_s seconds."""
    t0 = time.perf_counter()
    solve(1)
    one = time.perf_counter() - t0
    iters = int(max(2, min(max_iters, budget_s / max(one, 1e-4))))
    t0 = time.perf_counter()
    solve(iters)
    dt = time.perf_counter() - t0
    return iters, dt, unit_per_iter * iters / dt


def cpu_baseline_dense(w, eps, label, budget_s=12.0):
    import oracle
    threads = oracle.max_threads()
    run = lambda it: oracle.solve(w.a, w.b, eps, it, tol=1e-30, check_every=10, C=w.C)
    iters, dt, rate = _oracle_rate(run, budget_s, 1.0)
    oracle.set_threads(1)
    try:
        t0 = time.perf_counter()
        run(2 if w.n * w.m > 1 << 22 else 20)
        dt1 = (time.perf_counter() - t0) / (2 if w.n * w.m > 1 << 22 else 20)
    finally:
        oracle.set_threads(threads)
    return {"value": rate, "unit": "iter/s", "cores": threads, "kind": "oracle",
            "sample": f"{iters} iterations of Alg. 1 (check every 10) on the same {label} inputs, fp64, "
                      f"OpenMP over rows/columns, {dt:.1f} s",
            "one_thread_value": 1.0 / dt1}


def cpu_baseline_points(w, label, sub, budget_s=12.0):
    """Point clouds: the oracle on the first `sub` points of each cloud (all of them when sub is None)."""
    import numpy as np
    import oracle
    X, Y, a, b = w.X, w.Y, w.a, w.b
    if sub is not None and sub < w.n:
        X, Y = np.ascontiguousarray(X[:sub]), np.ascontiguousarray(Y[:sub])
        a = np.ascontiguousarray(a[:sub] / a[:sub].sum(dtype=np.float64)).astype(np.float32)
        b = np.ascontiguousarray(b[:sub] / b[:sub].sum(dtype=np.float64)).astype(np.float32)
    pairs = 2.0 * X.shape[0] * Y.shape[0]
    run = lambda it: oracle.solve(a, b, w.eps, it, tol=1e-30, check_every=10, X=X, Y=Y)
    iters, dt, rate = _oracle_rate(run, budget_s, pairs / 1e9, max_iters=50)
    return {"value": rate, "unit": "Gpair/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"{iters} iterations of Alg. 1 on {'the first %d points of each cloud of ' % sub if sub else ''}"
                      f"the same {label} inputs, fp64, {dt:.1f} s"}


# Point-cloud LSE pass, optimistic variant, per point pair: d fp64 FMAs, one fp64 subtraction, one
# fp64 -> fp32 conversion and one fp32 addition at 4 issue cycles per wave64 instruction, v_exp_f32 at
# 8; counted as 2d + 1 fp64 and 2 fp32 floating-point operations.  1024 SIMDs at 2.4 GHz.
def points_alu_peak(d):
    cycles_per_wave_pair = 4 * (d + 3) + 8
    pairs_per_s = 1024 * 2.4e9 * 64 / cycles_per_wave_pair
    flop_per_pair = 2 * d + 3
    return pairs_per_s, flop_per_pair


def _spin_up(torch, kind, ms, solve):
    """Brings the device from idle to its sustained clocks before anything is timed.  An idle MI355X runs the
    first milliseconds of a compute-heavy kernel slower: the same 100-iteration c2 solve takes 51.3 us per
    iteration after 0.5 s of idle, 49.5 after 100 - 400 ms of plain copies (memory traffic alone does not raise
    the shader clock), 47.6 right after 25 ms or more of the solver's own work, and 50.6 again after 20 ms of
    idle.  kind = "solver": untimed solves of the same problem for `ms` milliseconds; "copies": device-to-device
    copies; "none".  Not part of any timed region, and separate from the W warm-up steps, which still run."""
    if ms <= 0 or kind == "none":
        return
    t0 = time.perf_counter()
    if kind == "copies":
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(8):
                dst.copy_(src)
            torch.cuda.synchronize()
        return
    while (time.perf_counter() - t0) * 1e3 < ms:
        solve()
        torch.cuda.synchronize()


def _solve_timed(fs, torch, a, b, eps, steps, tol, warmup, time_kernels=True, spinup=("none", 0.0), **geo_kw):
    n, m = a.shape[0], b.shape[0]
    f = torch.empty(n, dtype=torch.float32, device="cuda")
    g = torch.empty(m, dtype=torch.float32, device="cuda")
    _spin_up(torch, spinup[0], spinup[1],
             lambda: fs.fs_sinkhorn_solve(a, b, eps, max(1, min(200, steps)), 0.0, f=f, g=g, **geo_kw))
    # warm-up: W untimed iterations (also sizes the library's cached workspace)
    fs.fs_sinkhorn_solve(a, b, eps, warmup, 0.0, f=f, g=g, **geo_kw)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    r = fs.fs_sinkhorn_solve(a, b, eps, steps, tol, f=f, g=g, **geo_kw)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if time_kernels:
        # The dominant kernel's own duration comes from the SAME solve run once more, right away, with its launches
        # stamped by HIP events: a stamped dispatch costs 10 - 50 us of queue and host time, which at 20 iterations
        # (one launch) would be 2 - 5 % of the very time being reported.  Same inputs, same iteration count, same
        # kernels (the results are bit-identical); fs_last_kernel_timing() reads the events afterwards.
        r2 = fs.fs_sinkhorn_solve(a, b, eps, steps, tol, f=f, g=g, time_kernel_every=1, **geo_kw)
        torch.cuda.synchronize()
        assert r2["iters"] == r["iters"]
    return r, dt


def bench_dense(args, name):
    import torch
    from paper_2605_00837_amd import binding as fs, workloads as W

    torch.cuda.set_device(0)
    if name == "c1":
        w = W.c1_small_dense()
        eps, steps_default, tol, label = w.eps, 200, 0.0, "c1_dense_uniform2d n=m=256"
        desc = "uniform weights, eps=0.05, 200 fixed iterations"
        metric = "sinkhorn_iters_per_sec_dense_n256_fp32_eps5e-2"
    elif name == "c2":
        w = W.c2_dense_gauss(args.n)
        eps, steps_default, tol, label = w.eps, 1000, w.tol, f"c2_dense_gauss2d n=m={w.n}"
        desc = "Dirichlet(1) weights, eps=1e-2, tol=1e-6, check_every=10"
        metric = ("sinkhorn_iters_per_sec_dense_n8192_fp32_eps1e-2" if w.n == 8192
                  else f"sinkhorn_iters_per_sec_dense_n{w.n}_fp32_eps1e-2")
    elif name == "c3":
        w = W.c3_small_eps()
        eps = w.eps_list[args.eps_index]
        steps_default, tol, label = 2000, 0.0, "c3_small_eps_sweep n=m=4096"
        desc = f"uniform weights, cost / max cost, eps={eps:g}, 2000 fixed iterations"
        metric = f"sinkhorn_iters_per_sec_dense_n4096_fp32_eps{eps:.0e}"
    else:                                                     # c5d: the dense variant of the colour workload
        w = W.c5_colour(16384, args.m5, dense=True)
        w.X = w.Y = None
        eps, steps_default, tol, label = w.eps, w.max_iter, w.tol, f"c5_colour_rgb dense 16384 x {args.m5}"
        desc = "Dirichlet(2) weights, eps=5e-3, tol=1e-5, check_every=10, C built from the RGB points"
        metric = f"sinkhorn_iters_per_sec_dense_16384x{args.m5}_fp32_eps5e-3"
    n, m = w.n, w.m
    steps = args.steps if args.steps > 0 else steps_default
    C, a, b = (torch.from_numpy(t).cuda() for t in (w.C, w.a, w.b))
    esize = 4
    if args.cost_dtype != "f32":      # C stored in 2 bytes per entry (the arithmetic stays what it is): not the headline
        C = C.to(torch.float16 if args.cost_dtype == "f16" else torch.bfloat16)
        esize = 2
    kw = dict(C=C, kernel_mode=args.kernel_mode, fused_variant=args.fused_variant)
    if tol > 0.0:
        kw["check_every"] = 10
    # the kernels that run a whole solve in one launch cannot be sampled per iteration (asking for it would
    # make the library take the multi-kernel path instead): they are timed by the wall clock alone
    choice = fs.fs_kernel_choice(n, m, kernel_mode=args.kernel_mode, fused_variant=args.fused_variant)
    one_launch_kernel = choice in ("small", "coop", "grid")
    r, dt = _solve_timed(fs, torch, a, b, eps, steps, tol, args.warmup, time_kernels=not one_launch_kernel,
                         spinup=(args.spinup, args.spinup_ms), **kw)
    iters = r["iters"]
    kern_ms, launches, kern_name, covered = (0.0, 0, "k_" + choice, 0) if one_launch_kernel else fs.fs_last_kernel_timing()

    # Algorithmic bytes.  One pass over C with V in and F, U out is what one iteration of a kernel that fuses the
    # two half-steps needs; two passes (the row pass and the column pass each read C) is the floor of any two-kernel
    # iteration and the figure the survey of the paper's method states.  Nothing is credited above the one-pass figure.
    bytes_one_pass = n * m * esize + m * 8 + n * 16
    bytes_two_pass = 2 * n * m * esize
    per_iter_ms = kern_ms * launches / max(covered, 1)
    alg_bytes_launch = bytes_one_pass * (covered / max(launches, 1)) if not one_launch_kernel else None
    out = {
        "metric": metric if esize == 4 else metric.replace("_fp32_", f"_{args.cost_dtype}cost_"),
        "value": iters / dt, "unit": "iter/s", "n_gpus": 1, "steps": iters, "warmup": args.warmup,
        "ms_per_step": dt * 1e3 / max(iters, 1), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{label} {args.cost_dtype} C ({n * m * esize / 2 ** 20:g} MiB), {desc}, max_iter={steps}",
                   "kernel_path": kern_name, "potentials": "fp64 internal, fp32 out",
                   "spinup": f"{args.spinup} {args.spinup_ms:g} ms"},
        "ms_to_stop": dt * 1e3, "converged": r["converged"], "marginal_err": r["marginal_err"],
    }
    if alg_bytes_launch is not None and launches > 0:
        achieved = alg_bytes_launch / (kern_ms * 1e-3) / 1e9
        traffic, src = _traffic_from_profiles(kern_name, n, m)
        out["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                           "traffic_source": (src + " (rocprofv3 --pmc runs of their own, not this run; FETCH_SIZE + "
                                                    "WRITE_SIZE count L2 <-> fabric bytes, served by the memory-side "
                                                    "cache or by HBM alike)") if src else None,
                           "kernel": kern_name, "kernel_avg_us": kern_ms * 1e3, "kernel_launches_timed": launches,
                           "kernel_timing": "HIP events stamped with the start and stop of the dispatch, in a repeat of "
                                            "the timed solve run right after it (stamping costs queue time)",
                           "iterations_per_launch": covered / max(launches, 1), "kernel_us_per_iteration": per_iter_ms * 1e3,
                           "algorithmic_bytes_per_launch": alg_bytes_launch}
        rows_pp = 64 if m <= 256 else 32 if m <= 512 else 16 if m <= 1024 else 8 if m <= 2048 else 4 if m <= 4096 else 2   # rows per panel of k_resident
        panels = -(-n // rows_pp)
        wgs = min(torch.cuda.get_device_properties(0).multi_processor_count, panels, 256)
        if kern_name == "k_resident" and panels > 4 * wgs:
            per_wg = -(-panels // wgs)
            out["roofline"]["resident"] = {
                "note": "four of the %d panels of every workgroup are not fetched in an iteration: two stay in registers "
                        "for a whole launch, and the two a pass ends with stay in LDS as the first two of the next pass "
                        "(the sweep turns round): %.3f of C is read from memory per iteration; achieved / frac are the "
                        "algorithmic bytes (all of C) over time, as for any other kernel" % (per_wg, 1.0 - 4.0 / per_wg)}
        elif kern_name == "k_resident":
            # C stays in LDS and registers for a whole launch: the algorithmic bytes above are NOT read from memory
            # (achieved / frac say how this compares with a pass that would stream them).  What bounds the pass is
            # vector-ALU issue: 8 issue slots per entry (cvt, fma64, add64, cvt, v_exp_f32 = 2, add, fma) of 4 cycles
            # per wave instruction on 1024 SIMDs at 2.4 GHz.
            peak_entries = 1024 * 2.4e9 * 64 / (8 * 4)
            ach_entries = n * m / (per_iter_ms * 1e-3)
            out["roofline"]["resident"] = {
                "note": "the workgroups hold C in LDS and registers for a whole launch: nothing of size n x m is read "
                        "from memory inside an iteration; the pass is bound by vector-ALU issue, the iteration by the "
                        "pass plus the grid-wide exchange",
                "bound": "alu", "achieved": ach_entries, "peak": peak_entries, "unit": "entries/s",
                "frac": ach_entries / peak_entries}
    else:
        # the whole solve runs inside one launch that keeps C in registers: latency-bound, no roofline fraction claimed
        out["roofline"] = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                           "traffic": None, "kernel": kern_name, "note": "launch- and latency-bound "
                           "size: C is read once per solve and stays in registers; microseconds per iteration is the figure"}
    it_gbs = bytes_one_pass * iters / dt / 1e9
    out["iteration"] = {"bytes_one_pass": bytes_one_pass, "bytes_two_pass_survey": bytes_two_pass,
                        "achieved_GBs": it_gbs, "frac_iteration": it_gbs / HBM_PEAK_GBS,
                        "two_pass_equivalent_GBs": bytes_two_pass * iters / dt / 1e9,
                        "us_per_iteration": dt * 1e6 / max(iters, 1)}
    if not args.no_cpu_baseline and esize == 4:
        out["cpu_baseline"] = cpu_baseline_dense(w, eps, label, budget_s=12.0 if n * m >= 1 << 20 else 3.0)
    print(json.dumps(out))


def bench_points(args, name):
    import torch
    from paper_2605_00837_amd import binding as fs, workloads as W

    torch.cuda.set_device(0)
    if name == "c4":
        w = W.c4_sphere_points(args.n if args.n != 8192 else 65536)
        steps_default, tol = w.max_iter, 0.0
        label = f"c4_sphere_points n=m={w.n} d=3"
        desc = f"eps={w.eps:g}, uniform weights, fixed iterations"
        sub = 16384
    else:
        w = W.c5_colour(16384, args.m5)
        steps_default, tol = w.max_iter, w.tol
        label = f"c5_colour_rgb points 16384 x {args.m5} d=3"
        desc = f"eps={w.eps:g}, Dirichlet(2) weights, tol=1e-5, check_every=10"
        sub = None
    n, m, d = w.n, w.m, w.X.shape[1]
    steps = args.steps if args.steps > 0 else steps_default
    X, Y, a, b = (torch.from_numpy(t).cuda() for t in (w.X, w.Y, w.a, w.b))
    kw = dict(X=X, Y=Y)
    if tol > 0.0:
        kw["check_every"] = 10
    r, dt = _solve_timed(fs, torch, a, b, w.eps, steps, tol, args.warmup, spinup=(args.spinup, args.spinup_ms), **kw)
    iters = r["iters"]
    kern_ms, launches, kern_name, covered = fs.fs_last_kernel_timing()
    peak_pairs, flop_per_pair = points_alu_peak(d)
    pairs_per_s = n * m / (kern_ms * 1e-3)
    achieved = pairs_per_s * flop_per_pair / 1e12
    peak = peak_pairs * flop_per_pair / 1e12
    out = {
        "metric": f"sinkhorn_point_pairs_per_sec_{n}x{m}_d{d}", "value": 2.0 * n * m * iters / dt / 1e9, "unit": "Gpair/s",
        "n_gpus": 1, "steps": iters, "warmup": args.warmup, "ms_per_step": dt * 1e3 / max(iters, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{label}, {desc}, max_iter={steps}, cost recomputed per pair (never stored)",
                   "kernel_path": kern_name, "spinup": f"{args.spinup} {args.spinup_ms:g} ms"},
        "iters_per_sec": iters / dt, "ms_to_stop": dt * 1e3, "converged": r["converged"], "marginal_err": r["marginal_err"],
        "roofline": {"bound": "alu", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": None, "kernel": kern_name, "kernel_avg_us": kern_ms * 1e3, "kernel_launches_timed": launches,
                     "flop_per_pair": flop_per_pair, "pairs_per_launch": n * m,
                     "peak_note": "issue rate of this kernel's own instruction mix (d + 3 full-rate vector "
                                  "instructions and one v_exp_f32 per pair); the two fractions below are against the "
                                  "chip's plain fp64 vector peak and against its v_exp_f32 rate",
                     "fp64_vector": {"achieved_TFLOPs": pairs_per_s * (2 * d + 1) / 1e12, "peak_TFLOPs": FP64_VECTOR_PEAK_TFLOPS,
                                     "frac": pairs_per_s * (2 * d + 1) / 1e12 / FP64_VECTOR_PEAK_TFLOPS},
                     "v_exp_f32": {"achieved_per_s": pairs_per_s, "peak_per_s": EXP_PEAK_PER_S,
                                   "frac": pairs_per_s / EXP_PEAK_PER_S}},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_points(w, label, sub)
    print(json.dumps(out))


def calibrate_copy(mib=256, reps=5):
    import torch
    src = torch.empty(mib << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy_mib": mib, "copies": reps}))


def calibrate_read(sizes_mib=(64, 128, 256, 512, 1024), reps=20):
    """The practical read ceiling of the device: a plain streaming read kernel (fs_read_rate: one workgroup of 1024
    lanes per compute unit, 16-byte loads) over buffers of the sizes of the dense workloads, beside the published
    HBM peak.  One JSON line."""
    import torch
    from paper_2605_00837_amd import binding as fs
    torch.cuda.set_device(0)
    buf = torch.zeros(max(sizes_mib) << 20, dtype=torch.uint8, device="cuda")
    _spin_up(torch, "copies", 100.0, None)
    out = {"calibrate_read": "plain streaming read kernel, average of %d passes after 2 untimed ones" % reps,
           "hbm_peak_GBs": HBM_PEAK_GBS, "sizes": []}
    for mib in sizes_mib:
        us = min(fs.fs_read_rate(buf[: mib << 20], reps) for _ in range(3))
        out["sizes"].append({"MiB": mib, "us_per_pass": us, "GBs": (mib << 20) / (us * 1e-6) / 1e9,
                             "frac_of_peak": (mib << 20) / (us * 1e-6) / 1e9 / HBM_PEAK_GBS})
    print(json.dumps(out))


def bench_after_loop(args):
    """The entry points that follow a solve (Eq. 5 plan, cost of Alg. 1's last step, one-pass diagnostics,
    barycentric mapping of Sec. 5.6), timed end to end on the workload's inputs after a short solve:
    `reps` back-to-back calls between two synchronisations, all launches of a call included.  Prints one JSON
    object (not the headline line)."""
    import torch
    from paper_2605_00837_amd import binding as fs, workloads as W

    torch.cuda.set_device(0)
    name = args.workload
    if name in ("c4", "c5p"):
        w = W.c4_sphere_points(args.n if args.n != 8192 else 65536) if name == "c4" else W.c5_colour(16384, args.m5)
        geo = dict(X=torch.from_numpy(w.X).cuda(), Y=torch.from_numpy(w.Y).cuda())
        unit_bytes = None
    else:
        w = {"c1": W.c1_small_dense, "c2": lambda: W.c2_dense_gauss(args.n), "c3": W.c3_small_eps}.get(
            name, lambda: W.c5_colour(16384, args.m5, dense=True))()
        geo = dict(C=torch.from_numpy(w.C).cuda())
        unit_bytes = w.n * w.m * 4
    eps = w.eps_list[args.eps_index] if name == "c3" else w.eps
    a, b = torch.from_numpy(w.a).cuda(), torch.from_numpy(w.b).cuda()
    _spin_up(torch, "copies", args.spinup_ms, None)
    r = fs.fs_sinkhorn_solve(a, b, eps, 50, 0.0, **geo)
    f, g = r["f"], r["g"]
    Z = torch.rand(w.m, 3, device="cuda")
    calls = {"fs_cost": lambda: fs.fs_cost(a, b, eps, f, g, **geo),
             "fs_diagnostics": lambda: fs.fs_diagnostics(a, b, eps, f, g, **geo),
             "fs_barycentric_dz3": lambda: fs.fs_barycentric(a, b, eps, f, g, Z, **geo)}
    if unit_bytes is not None and w.m % 4 == 0:
        P = torch.empty(w.n, w.m, device="cuda")
        calls["fs_plan"] = lambda: fs.fs_plan(a, b, eps, f, g, P=P, **geo)
    reps = 20 if unit_bytes is not None else 5
    out = {"after_loop": name, "n": w.n, "m": w.m, "reps": reps, "us_per_call": {}}
    for key, fn in calls.items():
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / reps * 1e6
        out["us_per_call"][key] = us
        if unit_bytes is not None:
            nbytes = unit_bytes * (2 if key == "fs_plan" else 1)
            out.setdefault("frac_of_hbm_peak", {})[key] = nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS
        else:
            # in units of one LSE pass over all point pairs at that kernel's issue bound
            pairs_per_s, _ = points_alu_peak(w.X.shape[1])
            out.setdefault("lse_passes_equivalent", {})[key] = us * 1e-6 * pairs_per_s / (w.n * w.m)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", choices=["c1", "c2", "c3", "c4", "c5p", "c5d"], default="c2")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="iterations of the timed solve (0: the workload's own count)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--spinup", choices=["solver", "copies", "none"], default="solver",
                    help="what keeps the device busy before the warm-up solve (clock ramp from idle; untimed)")
    ap.add_argument("--spinup-ms", type=float, default=100.0, help="for how long, in milliseconds")
    ap.add_argument("--n", type=int, default=8192, help="c2 / c4: problem size (default: the workload's own)")
    ap.add_argument("--m5", type=int, default=16384, choices=[16384, 12288], help="c5: number of target points")
    ap.add_argument("--eps-index", type=int, default=1, help="c3: which of eps = 1e-1, 1e-2, 1e-3, 1e-4")
    ap.add_argument("--kernel-mode", type=int, default=0)
    ap.add_argument("--fused-variant", type=int, default=0)
    ap.add_argument("--cost-dtype", choices=["f32", "f16", "bf16"], default="f32",
                    help="dense workloads: storage type of C (2-byte types are widened exactly; not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--calibrate-read", action="store_true",
                    help="print the read rate a plain streaming kernel reaches on buffers of 64 MiB .. 1 GiB")
    ap.add_argument("--after-loop", action="store_true",
                    help="time fs_cost / fs_diagnostics / fs_plan / fs_barycentric on the workload instead of the solve")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        calibrate_copy()
    elif args.calibrate_read:
        calibrate_read()
    elif args.after_loop:
        bench_after_loop(args)
    elif args.workload in ("c4", "c5p"):
        bench_points(args, args.workload)
    else:
        bench_dense(args, args.workload)


if __name__ == "__main__":
    main()
