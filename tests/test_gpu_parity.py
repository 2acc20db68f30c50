"""GPU parity: the HIP path (through the C ABI binding) against the CPU oracle,
element by element on the same seeded inputs.

Tolerances (north-star): potentials max|df|/eps <= 1e-3 for the fp32 outputs,
plan-marginal L1 difference <= 1e-5, transport-cost relative error <= 1e-4.
The library carries the potentials in fp64 internally and can hand them out in
fp64; those are held to a much tighter bound (1e-5 in units of eps; the
difference to the oracle is then only the fp32 exp2/log2 and summation noise).
"""
import math

import numpy as np
import pytest

from paper_2605_00837_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-3       # max |df| / eps, fp32 outputs
TOL_F64 = 2e-5       # max |df| / eps, fp64 outputs
TOL_MARG = 1e-5      # L1 difference of plan marginals
TOL_COST = 1e-4      # relative


@pytest.fixture(scope="module")
def fs():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_00837_amd import binding
    return binding


def dev(x, dtype=None):
    import torch
    if x is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def to_dev(w):
    return dict(C=dev(w.C), X=dev(w.X), Y=dev(w.Y)), dev(w.a), dev(w.b)


def pot_err(x_gpu, x_ref, eps):
    return float(np.max(np.abs(np.asarray(x_gpu, dtype=np.float64) - x_ref)) / eps)


# ------------------------------------------------------------------ kernel level: one half-step
DENSE_SHAPES = [(1, 1), (2, 3), (3, 2), (63, 65), (64, 64), (65, 63), (255, 257), (257, 256), (100, 1028),
                (300, 1100), (37, 4100), (515, 2048)]


@pytest.mark.parametrize("n,m", DENSE_SHAPES)
def test_dense_half_steps(fs, oracle, n, m):
    import torch
    w = W.random_dense(n, m, seed=1000 + n * 7 + m, cmax=3.0, eps=0.02)
    rng = np.random.default_rng(n * 31 + m)
    g0 = rng.standard_normal(m) * 0.3
    f0 = rng.standard_normal(n) * 0.3
    geo, a, b = to_dev(w)
    f_gpu = fs.fs_update_f(a, b, w.eps, dev(g0), **geo).cpu().numpy()
    g_gpu = fs.fs_update_g(a, b, w.eps, dev(f0), **geo).cpu().numpy()
    f_ref = oracle.update_f(w.a, w.b, w.eps, g0, C=w.C)
    g_ref = oracle.update_g(w.a, w.b, w.eps, f0, C=w.C)
    assert pot_err(f_gpu, f_ref, w.eps) < TOL_F64
    assert pot_err(g_gpu, g_ref, w.eps) < TOL_F64


@pytest.mark.parametrize("n,m,d", [(1, 1, 1), (5, 7, 2), (257, 300, 3), (600, 513, 3), (300, 257, 4),
                                   (129, 200, 5), (70, 90, 17), (40, 33, 64)])
def test_points_half_steps(fs, oracle, n, m, d):
    w = W.random_points(n, m, d, seed=2000 + n + m + d, eps=0.02)
    rng = np.random.default_rng(n * 31 + m + d)
    g0 = rng.standard_normal(m) * 0.3
    f0 = rng.standard_normal(n) * 0.3
    geo, a, b = to_dev(w)
    f_gpu = fs.fs_update_f(a, b, w.eps, dev(g0), **geo).cpu().numpy()
    g_gpu = fs.fs_update_g(a, b, w.eps, dev(f0), **geo).cpu().numpy()
    f_ref = oracle.update_f(w.a, w.b, w.eps, g0, X=w.X, Y=w.Y)
    g_ref = oracle.update_g(w.a, w.b, w.eps, f0, X=w.X, Y=w.Y)
    assert pot_err(f_gpu, f_ref, w.eps) < TOL_F64
    assert pot_err(g_gpu, g_ref, w.eps) < TOL_F64


# ------------------------------------------------------------------ full solves, every kernel path
def _solve_and_compare(fs, oracle, w, iters, eps=None, **kw):
    eps = w.eps if eps is None else eps
    geo, a, b = to_dev(w)
    r = fs.fs_sinkhorn_solve(a, b, eps, iters, 0.0, want_f64=True, **geo, **kw)
    ref = oracle.solve(w.a, w.b, eps, iters, C=w.C, X=w.X, Y=w.Y)
    assert r["iters"] == iters and not r["nonfinite"]
    e64 = max(pot_err(r["f64"].cpu().numpy(), ref["f"], eps), pot_err(r["g64"].cpu().numpy(), ref["g"], eps))
    e32 = max(pot_err(r["f"].cpu().numpy(), ref["f"], eps), pot_err(r["g"].cpu().numpy(), ref["g"], eps))
    return r, ref, e64, e32


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("n,m", [(1, 4), (4, 4), (130, 64), (67, 1024), (517, 1028), (300, 4096), (90, 8192),
                                 (130, 2052), (40, 9000), (33, 12288), (30, 13004), (21, 16384),
                                 (70, 1027), (64, 4097), (45, 8190), (37, 8189), (20, 16383), (50, 3001),
                                 (2049, 4096), (2300, 1500), (2051, 1026)])     # many panels per workgroup
def test_dense_solve_modes(fs, oracle, mode, n, m):
    w = W.random_dense(n, m, seed=3000 + n + m, cmax=2.0, eps=0.03)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 25, kernel_mode=mode)
    assert e64 < TOL_F64 and e32 < TOL_F32
    # the trailing pass reports err of the last iterate
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


@pytest.mark.parametrize("variant", [0, 1])      # 0: one wave per row (k_fused_rows), 1: all lanes on columns (k_fused<256,1,4>)
@pytest.mark.parametrize("n,m", [(5001, 256), (4099, 200), (1000, 512), (777, 260), (9, 4), (300, 508), (3, 256),
                                 (17000, 64), (40000, 8)])
def test_fused_narrow(fs, oracle, variant, n, m):
    """Narrow matrices on the fused path: many panels per wave, ragged row counts, column counts on both sides of
    the one- and two-group limits, fewer panels than waves."""
    w = W.random_dense(n, m, seed=3500 + n + m, cmax=2.0, eps=0.04)
    w.a[::7] = 0.0
    w.a[:] = w.a / w.a.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 15, kernel_mode=2, fused_variant=variant)
    fin = np.isfinite(ref["f"])
    assert np.array_equal(np.isfinite(r["f64"].cpu().numpy()), fin)
    assert pot_err(r["f64"].cpu().numpy()[fin], ref["f"][fin], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4])
def test_fused_variants_full_width(fs, oracle, variant):
    w = W.random_dense(70, 8192, seed=77, cmax=2.0, eps=0.03)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 12, kernel_mode=2, fused_variant=variant)
    assert e64 < TOL_F64 and e32 < TOL_F32


def test_fused_column_repair_path(fs, oracle):
    """fused_variant >= 100 is a test knob: it shifts the predicted column references of the fused
    pass far too high, so that every column's partial sums underflow and the combine kernel has to
    recompute every column exactly from C.  The results must not change."""
    w = W.random_dense(70, 8192, seed=78, cmax=2.0, eps=0.03)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 9, kernel_mode=2, fused_variant=100)
    assert e64 < TOL_F64 and e32 < TOL_F32
    w = W.random_dense(300, 4100, seed=79, cmax=2.0, eps=0.03)       # odd tail columns on the same path
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 9, kernel_mode=2, fused_variant=100)
    assert e64 < TOL_F64 and e32 < TOL_F32
    for n, m in ((64, 3000), (50, 4096), (35, 10000), (25, 16384), (40, 8191), (33, 2050), (2100, 4096), (2064, 3001)):  # other widths
        w = W.random_dense(n, m, seed=80 + m, cmax=2.0, eps=0.03)
        r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 9, kernel_mode=2, fused_variant=100)
        assert e64 < TOL_F64 and e32 < TOL_F32, (n, m, e64, e32)


# ------------------------------------------------------------------ cost matrix stored in 2 bytes per entry
def _rounded_cost(C, dtype_name):
    """The fp32 values of C after rounding to fp16 / bfloat16 (what the oracle is given), and the device
    tensor in that storage type.  The rounding is torch's conversion, on the CPU."""
    import torch
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[dtype_name]
    t16 = torch.from_numpy(np.ascontiguousarray(C)).to(tdt)
    return t16.to(torch.float32).numpy(), t16.cuda()


@pytest.mark.parametrize("dtype_name", ["f16", "bf16"])
@pytest.mark.parametrize("n,m,mode,variant", [
    (300, 520, 1, 0), (70, 8, 1, 0), (3, 2040, 0, 0),          # streaming kernels (automatic up to m = 2048)
    (130, 4096, 2, 0), (90, 8192, 2, 0), (45, 6008, 2, 0),     # prefetch kernel, 8 columns per lane
    (33, 10000, 2, 0), (21, 16384, 2, 0),                      # two groups of 8 columns per lane
    (70, 8192, 2, 100), (35, 10000, 2, 100), (64, 3000, 2, 100),   # optimistic from the start: repair from 2-byte C
    (40, 20000, 0, 0)])                                        # wider than the fused kernels: streaming
def test_dense_solve_half_precision_cost(fs, oracle, dtype_name, n, m, mode, variant):
    """C stored as fp16 / bfloat16: the solve must be the fp32 solve on the rounded matrix (the oracle gets
    the rounded values), to the same tolerances as every other dense path."""
    w = W.random_dense(n, m, seed=3300 + n + m, cmax=2.0, eps=0.03)
    C32, C16 = _rounded_cost(w.C, dtype_name)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, 25, 0.0, C=C16, want_f64=True, kernel_mode=mode,
                             fused_variant=variant)
    ref = oracle.solve(w.a, w.b, w.eps, 25, C=C32)
    assert r["iters"] == 25 and not r["nonfinite"]
    e64 = max(pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps), pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps))
    e32 = max(pot_err(r["f"].cpu().numpy(), ref["f"], w.eps), pot_err(r["g"].cpu().numpy(), ref["g"], w.eps))
    assert e64 < TOL_F64 and e32 < TOL_F32, (e64, e32)
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=C32))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7
    # and it is NOT the solve on the unrounded matrix: the result is closer to the oracle on the rounded one
    ref_full = oracle.solve(w.a, w.b, w.eps, 25, C=w.C)
    assert pot_err(r["f64"].cpu().numpy(), ref_full["f"], w.eps) > 2 * e64


@pytest.mark.parametrize("dtype_name", ["f16", "bf16"])
@pytest.mark.parametrize("n,m,mode", [(100, 120, 3), (64, 64, 0), (256, 256, 4), (300, 408, 0), (1000, 1024, 5),
                                      (900, 1200, 0)])
def test_one_launch_kernels_take_half_precision_cost(fs, oracle, dtype_name, n, m, mode):
    """The one-launch kernels widen a 2-byte C once, when they load their register tile."""
    if mode == 5:
        _needs_whole_chip()
    w = W.random_dense(n, m, seed=3500 + n + m, cmax=2.0, eps=0.03)
    C32, C16 = _rounded_cost(w.C, dtype_name)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, 25, 0.0, C=C16, want_f64=True, kernel_mode=mode)
    ref = oracle.solve(w.a, w.b, w.eps, 25, C=C32)
    assert r["iters"] == 25 and not r["nonfinite"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64


def test_batched_solves_take_half_precision_cost(fs, oracle):
    import torch
    B, n, m = 5, 96, 104
    rng = np.random.default_rng(3600)
    C = rng.uniform(0.0, 2.0, size=(B, n, m)).astype(np.float32)
    a = np.full((B, n), 1.0 / n, dtype=np.float32)
    b = np.full((B, m), 1.0 / m, dtype=np.float32)
    C16 = torch.from_numpy(C).to(torch.bfloat16)
    out = fs.fs_sinkhorn_dense_batched(C16.cuda(), dev(a), dev(b), 0.05, 20, 0.0, want_f64=True)
    res = fs.results_from_device(out["result"])
    C32 = C16.to(torch.float32).numpy()
    for p in range(B):
        ref = oracle.solve(a[p], b[p], 0.05, 20, C=C32[p])
        assert res[p]["iters"] == 20
        assert pot_err(out["f64"][p].cpu().numpy(), ref["f"], 0.05) < TOL_F64


def test_half_precision_cost_async_and_rejections(fs, oracle):
    import torch
    w = W.random_dense(60, 4096, seed=3401, cmax=2.0, eps=0.03)
    C32, C16 = _rounded_cost(w.C, "f16")
    h = fs.fs_sinkhorn_dense_ex(C16, dev(w.a), dev(w.b), w.eps, 15, 0.0)
    res = h.result()
    ref = oracle.solve(w.a, w.b, w.eps, 15, C=C32)
    assert res["iters"] == 15
    assert pot_err(h.f.cpu().numpy(), ref["f"], w.eps) < TOL_F32
    # rows that are not whole 16-byte chunks, the single-workgroup and batched kernels, point clouds
    a, b = dev(w.a), dev(np.full(4100, 1.0 / 4100, dtype=np.float32))
    with pytest.raises(fs.FsError, match="m % 8"):
        fs.fs_sinkhorn_solve(a, b, 0.1, 3, 0.0, C=torch.zeros(60, 4100, dtype=torch.float16, device="cuda"))
    u = torch.full((64,), 1 / 64, device="cuda")
    with pytest.raises(fs.FsError, match="dense cost matrix only"):
        fs.fs_sinkhorn_solve(u, u, 0.1, 3, 0.0, X=torch.zeros(64, 2, device="cuda"),
                             Y=torch.zeros(64, 2, device="cuda"), cost_dtype=1)
    with pytest.raises(fs.FsError, match="2048 < m"):
        fs.fs_sinkhorn_solve(u, torch.full((1024,), 1 / 1024, device="cuda"), 0.1, 3, 0.0,
                             C=torch.zeros(64, 1024, dtype=torch.bfloat16, device="cuda"), kernel_mode=2)


def _sweep_cases():
    """Seeded sweep over the widths where the dense driver changes kernels (and their neighbours), every kernel
    mode that takes the shape, all three storage types of C, occasional zero weights."""
    rng = np.random.default_rng(20240607)
    edges = [128, 256, 512, 1024, 2048, 4096, 8192, 12288, 16384]
    cases = []
    for t in range(48):
        if t % 3 == 0:
            m = int(rng.choice(edges)) + int(rng.choice([-8, -1, 0, 1, 8]))
        else:
            m = int(rng.integers(1, 17000))
        n = int(rng.integers(1, 400)) if m > 2048 else int(rng.integers(1, 1200))
        dt = ["f32", "f32", "f16", "bf16"][int(rng.integers(0, 4))] if m % 8 == 0 else "f32"
        modes = [0, 1]
        if dt == "f32" and (m <= 16384 and (m > 1024 or m % 4 == 0)):
            modes.append(2)
        if dt != "f32" and 2048 < m <= 16384:
            modes.append(2)
        if dt == "f32" and n <= 1024 and m <= 1024:
            modes.append(4)
        if dt == "f32" and n <= 256 and m <= 256:
            modes.append(3)
        mode = int(rng.choice(modes))
        eps = float(rng.choice([0.02, 0.05, 0.3]))
        cases.append((t, n, m, dt, mode, eps, bool(rng.integers(0, 3) == 0)))
    return cases


@pytest.mark.parametrize("t,n,m,dt,mode,eps,zeros", _sweep_cases())
def test_dense_shape_sweep(fs, oracle, t, n, m, dt, mode, eps, zeros):
    w = W.random_dense(n, m, seed=9100 + t, cmax=2.0, eps=eps)
    if zeros and n > 4 and m > 4:
        w.a[1::5] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
        w.b[3::7] = 0.0
        w.b[:] = w.b / w.b.sum(dtype=np.float64)
    if dt == "f32":
        C32, Cd = w.C, dev(w.C)
    else:
        C32, Cd = _rounded_cost(w.C, dt)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), eps, 12, 0.0, C=Cd, want_f64=True, kernel_mode=mode)
    ref = oracle.solve(w.a, w.b, eps, 12, C=C32)
    assert r["iters"] == 12 and not r["nonfinite"]
    fin_f, fin_g = np.isfinite(ref["f"]), np.isfinite(ref["g"])
    f64, g64 = r["f64"].cpu().numpy(), r["g64"].cpu().numpy()
    assert np.array_equal(np.isfinite(f64), fin_f) and np.array_equal(np.isfinite(g64), fin_g)
    assert pot_err(f64[fin_f], ref["f"][fin_f], eps) < TOL_F64
    assert pot_err(g64[fin_g], ref["g"][fin_g], eps) < TOL_F64


def test_dense_tall_full_width(fs, oracle):
    """8192 rows or more at m = 4096: the fused pass runs two workgroups per compute unit (512 sets of column
    partials); the row count is ragged against both the panel size and the grid."""
    n, m, eps = 8201, 4096, 0.05
    w = W.random_dense(n, m, seed=9300, cmax=2.0, eps=eps)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), eps, 6, 0.0, C=dev(w.C), want_f64=True)
    ref = oracle.solve(w.a, w.b, eps, 6, C=w.C)
    assert r["iters"] == 6 and not r["nonfinite"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], eps) < TOL_F64


def _points_sweep_cases():
    rng = np.random.default_rng(20240608)
    dims = [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64]
    cases = []
    for t in range(32):
        d = dims[t % len(dims)]
        n, m = int(rng.integers(1, 2500)), int(rng.integers(1, 2500))
        cases.append((t, n, m, d, float(rng.choice([0.02, 0.05, 0.3])), bool(rng.integers(0, 3) == 0)))
    return cases


@pytest.mark.parametrize("t,n,m,d,eps,zeros", _points_sweep_cases())
def test_points_shape_sweep(fs, oracle, t, n, m, d, eps, zeros):
    """Seeded sweep over every coordinate count the point-cloud kernels specialise on (vector kernels up to 4,
    matrix-core tiles of 8, 16, 32, 64 and their neighbours), ragged sizes, occasional zero weights."""
    w = W.random_points(n, m, d, seed=9300 + t, eps=eps)
    if zeros and n > 4 and m > 4:
        w.a[1::5] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
        w.b[3::7] = 0.0
        w.b[:] = w.b / w.b.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 10)
    assert e64 < TOL_F64 and e32 < TOL_F32, (e64, e32)
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], X=w.X, Y=w.Y))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


@pytest.mark.parametrize("n,m,dt", [(300, 20000, "f32"), (17, 16391, "f32"), (100, 24576, "f16"), (64, 32768, "bf16"),
                                    (1, 9000, "f32"), (1023, 8192, "f32"), (1024, 8192, "f32"), (700, 8190, "f32")])
def test_dense_short_wide_row_pass(fs, oracle, n, m, dt):
    """Few rows, many columns, streaming kernels: the row pass cut into column ranges (with a ragged last range, odd
    widths, 2-byte costs), and its neighbours that are not cut (1024 rows; fewer than two ranges of 4096 columns)."""
    eps = 0.05
    w = W.random_dense(n, m, seed=9700 + n + m, cmax=2.0, eps=eps)
    if n > 8:
        w.a[2::9] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    C32, Cd = (w.C, dev(w.C)) if dt == "f32" else _rounded_cost(w.C, dt)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), eps, 9, 0.0, C=Cd, want_f64=True, kernel_mode=1)
    ref = oracle.solve(w.a, w.b, eps, 9, C=C32)
    assert r["iters"] == 9 and not r["nonfinite"]
    fin = np.isfinite(ref["f"])
    f64, g64 = r["f64"].cpu().numpy(), r["g64"].cpu().numpy()
    assert np.array_equal(np.isfinite(f64), fin)
    assert pot_err(f64[fin], ref["f"][fin], eps) < TOL_F64
    assert pot_err(g64, ref["g"], eps) < TOL_F64
    err_ref = float(oracle.marginal_err(w.a, w.b, eps, ref["f"], ref["g"], C=C32))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


def _after_loop_sweep_cases():
    rng = np.random.default_rng(20240609)
    cases = []
    for t in range(40):
        if t % 2 == 0:
            kind, d = "dense", 0
            n, m = int(rng.integers(1, 2500)), int(rng.integers(1, 2500))
        else:
            kind, d = "points", int(rng.choice([1, 2, 3, 4, 5, 16]))
            if t % 8 == 1:                               # 8192 rows or more on one side: four rows per lane
                n, m = int(rng.integers(8192, 9500)), int(rng.integers(1, 400))
                if rng.integers(0, 2):
                    n, m = m, n
            else:
                n, m = int(rng.integers(1, 3000)), int(rng.integers(1, 3000))
        cases.append((t, kind, n, m, d, float(rng.choice([0.03, 0.1, 0.5])), int(rng.integers(1, 5)),
                      "f64" if rng.integers(0, 2) else "f32", bool(rng.integers(0, 3) == 0)))
    return cases


@pytest.mark.parametrize("t,kind,n,m,d,eps,dz,precision,zeros", _after_loop_sweep_cases())
def test_after_loop_shape_sweep(fs, oracle, t, kind, n, m, d, eps, dz, precision, zeros):
    """Seeded sweep of fs_diagnostics, fs_cost, fs_barycentric and fs_plan over ragged shapes on both sides of every
    launch-shape switch (single workgroup, one or four rows per lane, matrix-core tiles), unconverged potentials."""
    import torch
    w = W.random_dense(n, m, seed=9500 + t, cmax=2.0, eps=eps) if kind == "dense" else \
        W.random_points(n, m, d, seed=9500 + t, eps=eps)
    if zeros and n > 3 and m > 3:
        w.a[::3] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    ref = oracle.solve(w.a, w.b, eps, 3, C=w.C, X=w.X, Y=w.Y)
    f_h, g_h = ref["f"], ref["g"]
    dt = torch.float64
    if precision == "f32":
        f_h, g_h = f_h.astype(np.float32).astype(np.float64), g_h.astype(np.float32).astype(np.float64)
        dt = torch.float32
    geo, a, b = to_dev(w)
    fd, gd = dev(f_h, dt), dev(g_h, dt)
    r = fs.fs_diagnostics(a, b, eps, fd, gd, want_marginals=True, **geo)
    got = dict(zip(fs.DIAG_FIELDS, r["out"].cpu().numpy()))
    o = oracle.objectives(w.a, w.b, eps, f_h, g_h, C=w.C, X=w.X, Y=w.Y)
    ro, co = oracle.marginals(w.a, w.b, eps, f_h, g_h, C=w.C, X=w.X, Y=w.Y)
    for key in ("cost", "mass", "kl", "primal", "dual"):
        assert abs(got[key] - float(o[key])) <= 2e-6 * max(1.0, abs(float(o[key]))), (key, got[key], float(o[key]))
    assert np.abs(r["row_marginal"].cpu().numpy() - ro).sum() <= 2e-6
    assert np.abs(r["col_marginal"].cpu().numpy() - co).sum() <= 2e-6
    cost2 = float(fs.fs_cost(a, b, eps, fd, gd, **geo).cpu()[0])
    assert abs(cost2 - float(o["cost"])) <= 2e-6 * max(1.0, abs(float(o["cost"])))
    Z = np.random.default_rng(t).standard_normal((m, dz)).astype(np.float32)
    To = oracle.barycentric(w.a, w.b, eps, f_h, g_h, Z.astype(np.float64), C=w.C, X=w.X, Y=w.Y)
    T = fs.fs_barycentric(a, b, eps, fd, gd, dev(Z), **geo).cpu().numpy()
    assert np.abs(T - To).max() <= 5e-6 * (1.0 + float(np.abs(Z).max()))
    if n * m <= 2_000_000:
        P = fs.fs_plan(a, b, eps, fd, gd, **geo).cpu().numpy()
        Po = oracle.plan(w.a, w.b, eps, f_h, g_h, C=w.C, X=w.X, Y=w.Y)
        assert np.abs(P - Po).sum() <= 1e-5


@pytest.mark.parametrize("n,m,mode", [(5000, 64, 0), (3000, 12, 1), (40, 20000, 0), (9, 16388, 0), (2, 70001, 1)])
def test_dense_extreme_aspect_ratios(fs, oracle, n, m, mode):
    """Very tall (many rows of the error sum per workgroup of the combine) and very wide (beyond the
    widths the fused kernels cover: streaming kernels, many column strips) problems."""
    w = W.random_dense(n, m, seed=3500 + n + m, cmax=2.0, eps=0.03)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 15, kernel_mode=mode)
    assert e64 < TOL_F64 and e32 < TOL_F32
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


@pytest.mark.parametrize("n,m,d", [(1, 1, 3), (1, 700, 2), (900, 1, 4), (130, 140, 64), (2500, 40, 1)])
def test_points_extreme_shapes(fs, oracle, n, m, d):
    w = W.random_points(n, m, d, seed=4300 + n + m + d, eps=0.05)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 25)
    assert e64 < TOL_F64 and e32 < TOL_F32


def test_streaming_rejects_nothing_and_fused_rejects_odd_m(fs):
    w = W.random_dense(8, 10, seed=5)
    geo, a, b = to_dev(w)
    fs.fs_sinkhorn_solve(a, b, w.eps, 3, 0.0, kernel_mode=1, **geo)
    w2 = W.random_dense(8, 9, seed=5)
    geo2, a2, b2 = to_dev(w2)
    with pytest.raises(fs.FsError) as e:
        fs.fs_sinkhorn_solve(a2, b2, w2.eps, 3, 0.0, kernel_mode=2, **geo2)
    assert e.value.status == fs.FS_ERR_UNSUPPORTED


@pytest.mark.parametrize("n,m,d", [(300, 257, 3), (1000, 777, 3), (64, 64, 2), (129, 200, 5), (50, 60, 11),
                                   (700, 900, 8), (1500, 400, 16), (300, 2000, 17), (520, 515, 32), (400, 300, 50)])
def test_points_solve(fs, oracle, n, m, d):
    w = W.random_points(n, m, d, seed=4000 + n + m + d, eps=0.02)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 30)
    assert e64 < TOL_F64 and e32 < TOL_F32


@pytest.mark.parametrize("n,m,d,zero", [(300, 257, 3, False), (2100, 1500, 2, False), (700, 3000, 4, True),
                                        (1030, 1030, 1, False), (900, 1100, 6, True), (333, 1500, 20, False),
                                        (260, 130, 64, False), (1000, 70, 33, False)])
def test_points_optimistic_pass_and_repair(fs, oracle, n, m, d, zero):
    """fused_variant = 100 makes the point-cloud LSE pass optimistic (previous potential as the
    reference, plain fp32 sums) from the first iteration on, while the potentials still move by
    hundreds of units: the combine kernel then has to find and recompute the rows whose sums
    under- or overflowed.  The results must not change."""
    w = W.random_points(n, m, d, seed=4100 + n + m + d, eps=0.004)
    if zero:
        w.a[::7] = 0.0
        w.b[3::5] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
        w.b[:] = w.b / w.b.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 40, fused_variant=100)
    assert e64 < TOL_F64 and e32 < TOL_F32
    # the same solve on the device's own schedule (exact passes while the potentials move fast)
    r2, _, e64b, e32b = _solve_and_compare(fs, oracle, w, 40)
    assert e64b < TOL_F64 and e32b < TOL_F32


# ------------------------------------------------------------------ eps-scaling
@pytest.mark.parametrize("kind", ["dense", "points", "small"])
def test_annealed_regularisation(fs, oracle, kind):
    """fs_sinkhorn_annealed = the same chain of warm-started solves composed from the oracle (potentials
    handed from stage to stage as fp32, as the library does)."""
    if kind == "dense":
        w = W.random_dense(300, 520, seed=8100, cmax=1.0, eps=0.002)
    elif kind == "small":
        w = W.random_dense(90, 70, seed=8101, cmax=1.0, eps=0.002)
    else:
        w = W.random_points(400, 350, 3, seed=8102, eps=0.002)
    geo, a, b = to_dev(w)
    eps, eps0, decay, stage = w.eps, 0.25, 0.5, 8
    r = fs.fs_sinkhorn_annealed(a, b, eps, eps0, decay, stage, 30, 0.0, want_f64=True, **geo)
    f0 = g0 = None
    e = np.float32(eps0)
    nst = 0
    while e > np.float32(eps):
        o = oracle.solve(w.a, w.b, float(e), stage, C=w.C, X=w.X, Y=w.Y, f0=f0, g0=g0)
        f0 = o["f"].astype(np.float32).astype(np.float64)
        g0 = o["g"].astype(np.float32).astype(np.float64)
        e = np.float32(e * np.float32(decay))
        nst += 1
    o = oracle.solve(w.a, w.b, eps, 30, C=w.C, X=w.X, Y=w.Y, f0=f0, g0=g0)
    assert r["iters"] == 30 and r["total_iters"] == 30 + nst * stage
    # fp32 hand-over of potentials of size ~1 moves the start by ~1e-7/eps of the unit: allow for it
    assert pot_err(r["f64"].cpu().numpy(), o["f"], eps) < 2e-4 and pot_err(r["g64"].cpu().numpy(), o["g"], eps) < 2e-4
    assert pot_err(r["f"].cpu().numpy(), o["f"], eps) < TOL_F32
    err_ref = float(oracle.marginal_err(w.a, w.b, eps, o["f"], o["g"], C=w.C, X=w.X, Y=w.Y))
    assert abs(r["marginal_err"] - err_ref) <= 2e-3 * err_ref + 5e-7
    for bad in (dict(eps_start=eps / 2), dict(decay=1.0), dict(stage_iters=0)):
        kw = dict(eps_start=eps0, decay=decay, stage_iters=stage)
        kw.update(bad)
        with pytest.raises(fs.FsError):
            fs.fs_sinkhorn_annealed(a, b, eps, kw["eps_start"], kw["decay"], kw["stage_iters"], 5, 0.0, **geo)


# ------------------------------------------------------------------ single-workgroup kernel, batched solves
SMALL_SHAPES = [(1, 1), (1, 7), (5, 1), (31, 33), (64, 64), (100, 37), (128, 256), (256, 129), (256, 256), (200, 255)]


@pytest.mark.parametrize("n,m", SMALL_SHAPES)
def test_small_kernel_matches_oracle(fs, oracle, n, m):
    """kernel_mode = 3: the whole solve inside one workgroup (also what the automatic mode picks here)."""
    w = W.random_dense(n, m, seed=7000 + n + m, cmax=2.0, eps=0.02)
    if n > 8:
        w.a[2::9] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 40, kernel_mode=3)
    assert e64 < TOL_F64 and e32 < TOL_F32
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7
    # the multi-kernel path gives the same potentials (to rounding)
    r1, _, _, _ = _solve_and_compare(fs, oracle, w, 40, kernel_mode=1)
    assert float((r1["f64"] - r["f64"]).abs().max()) / w.eps < TOL_F64


def test_small_kernel_stop_rule_history_and_resume(fs, oracle):
    import torch
    w = W.random_dense(150, 190, seed=7100, cmax=1.0, eps=0.05)
    geo, a, b = to_dev(w)
    ref = oracle.solve(w.a, w.b, w.eps, 400, tol=1e-5, check_every=7, C=w.C, err_every_iter=True)
    hist = torch.full((400,), float("nan"), dtype=torch.float32, device="cuda")
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 400, 1e-5, C=geo["C"], want_f64=True, check_every=7, kernel_mode=3,
                             err_history=hist)
    assert r["converged"] and ref["converged"]
    assert abs(r["iters"] - int(ref["iters"])) <= 7 and r["iters"] % 7 == 0
    k = r["iters"]
    refk = oracle.solve(w.a, w.b, w.eps, k, C=w.C)
    assert pot_err(r["f64"].cpu().numpy(), refk["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), refk["g"], w.eps) < TOL_F64
    h = hist.cpu().numpy()
    eh = np.asarray(ref["err_hist"], dtype=np.float64)
    upto = min(k, int(ref["iters"]))
    assert np.all(np.isfinite(h[:upto]))
    assert np.allclose(h[:upto], eh[:upto], rtol=2e-3, atol=5e-7)
    assert np.all(np.isnan(h[k:]))
    # fixed count without the trailing error pass; resume from fp64 potentials = one longer run
    r1 = fs.fs_sinkhorn_solve(a, b, w.eps, 11, 0.0, C=geo["C"], want_f64=True, kernel_mode=3, skip_final_err=True)
    assert math.isnan(r1["marginal_err"]) and r1["iters"] == 11
    r2 = fs.fs_sinkhorn_solve(a, b, w.eps, 9, 0.0, C=geo["C"], want_f64=True, kernel_mode=3, warm_start=True,
                              f64_in=r1["f64"], g64_in=r1["g64"])
    r3 = fs.fs_sinkhorn_solve(a, b, w.eps, 20, 0.0, C=geo["C"], want_f64=True, kernel_mode=3)
    assert float((r2["f64"] - r3["f64"]).abs().max()) / w.eps < 1e-9
    assert float((r2["g64"] - r3["g64"]).abs().max()) / w.eps < 1e-9
    # max_iter = 0 returns the start
    r0 = fs.fs_sinkhorn_solve(a, b, w.eps, 0, 0.0, C=geo["C"], kernel_mode=3)
    assert r0["iters"] == 0 and float(r0["f"].abs().max()) == 0.0 and float(r0["g"].abs().max()) == 0.0


# ------------------------------------------------------------------ one launch over several workgroups (n, m <= 1024)
COOP_SHAPES = [(1, 1, 0), (5, 7, 0), (3, 1024, 0), (1024, 3, 0), (256, 256, 0), (257, 300, 0), (300, 257, 2),
               (129, 513, 1), (513, 129, 3), (700, 1000, 0), (1000, 700, 1), (1024, 1024, 0), (1024, 1024, 1),
               (512, 512, 0), (512, 512, 2), (64, 64, 3), (1023, 1021, 0)]


@pytest.mark.parametrize("n,m,variant", COOP_SHAPES)
def test_coop_kernel_matches_oracle(fs, oracle, n, m, variant):
    """kernel_mode = 4: the whole solve in one launch, rows split over up to 32 workgroups that exchange
    column partials once per iteration (fused_variant 1..3: fewer workgroups, more rows per lane)."""
    w = W.random_dense(n, m, seed=7500 + n + m, cmax=2.0, eps=0.02)
    if n > 8:
        w.a[2::9] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 30, kernel_mode=4, fused_variant=variant)
    assert e64 < TOL_F64 and e32 < TOL_F32, (e64, e32)
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


@pytest.mark.parametrize("n,m,d,variant", [(1, 1, 1, 0), (5, 7, 2, 0), (200, 200, 3, 0), (256, 256, 3, 1), (300, 257, 4, 0),
                                           (1024, 512, 3, 0), (512, 1024, 2, 0), (700, 500, 3, 0), (129, 513, 17, 2),
                                           (100, 90, 64, 0), (1000, 20, 5, 0)])
def test_coop_kernel_point_clouds(fs, oracle, n, m, d, variant):
    """kernel_mode = 4 on point clouds: the squared distances are formed once in fp64 (difference form) and
    stay in registers; everything else is the dense one-launch solver."""
    w = W.random_points(n, m, d, seed=7800 + n + m + d, eps=0.02)
    if n > 8:
        w.a[2::9] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 30, kernel_mode=4, fused_variant=variant)
    assert e64 < TOL_F64 and e32 < TOL_F32, (e64, e32)
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], X=w.X, Y=w.Y))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7
    # the multi-kernel point-cloud path (any other kernel_mode) agrees to rounding
    r1, _, _, _ = _solve_and_compare(fs, oracle, w, 30, kernel_mode=1)
    assert float((r1["f64"] - r["f64"]).abs().max()) / w.eps < TOL_F64


def test_coop_kernel_stop_rule_history_and_resume(fs, oracle):
    import torch
    w = W.random_dense(300, 410, seed=7600, cmax=1.0, eps=0.05)
    geo, a, b = to_dev(w)
    ref = oracle.solve(w.a, w.b, w.eps, 400, tol=1e-5, check_every=7, C=w.C, err_every_iter=True)
    hist = torch.full((400,), float("nan"), dtype=torch.float32, device="cuda")
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 400, 1e-5, C=geo["C"], want_f64=True, check_every=7, kernel_mode=4,
                             err_history=hist)
    assert r["converged"] and ref["converged"]
    assert abs(r["iters"] - int(ref["iters"])) <= 7 and r["iters"] % 7 == 0
    k = r["iters"]
    refk = oracle.solve(w.a, w.b, w.eps, k, C=w.C)
    assert pot_err(r["f64"].cpu().numpy(), refk["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), refk["g"], w.eps) < TOL_F64
    h = hist.cpu().numpy()
    eh = np.asarray(ref["err_hist"], dtype=np.float64)
    upto = min(k, int(ref["iters"]))
    assert np.all(np.isfinite(h[:upto]))
    assert np.allclose(h[:upto], eh[:upto], rtol=2e-3, atol=5e-7)
    assert np.all(np.isnan(h[k:]))
    # the multi-kernel driver stops at the same iteration with the same potentials (to rounding)
    rm = fs.fs_sinkhorn_solve(a, b, w.eps, 400, 1e-5, C=geo["C"], want_f64=True, check_every=7, kernel_mode=1)
    assert rm["iters"] == k and float((rm["f64"] - r["f64"]).abs().max()) / w.eps < TOL_F64
    # fixed count without the trailing error pass; resume from fp64 potentials = one longer run
    r1 = fs.fs_sinkhorn_solve(a, b, w.eps, 11, 0.0, C=geo["C"], want_f64=True, kernel_mode=4, skip_final_err=True)
    assert math.isnan(r1["marginal_err"]) and r1["iters"] == 11
    r2 = fs.fs_sinkhorn_solve(a, b, w.eps, 9, 0.0, C=geo["C"], want_f64=True, kernel_mode=4, warm_start=True,
                              f64_in=r1["f64"], g64_in=r1["g64"])
    r3 = fs.fs_sinkhorn_solve(a, b, w.eps, 20, 0.0, C=geo["C"], want_f64=True, kernel_mode=4)
    assert float((r2["f64"] - r3["f64"]).abs().max()) / w.eps < 1e-9
    assert float((r2["g64"] - r3["g64"]).abs().max()) / w.eps < 1e-9
    # repeated solves are bit-identical, and the asynchronous entry point runs the same kernel
    r4 = fs.fs_sinkhorn_solve(a, b, w.eps, 20, 0.0, C=geo["C"], want_f64=True, kernel_mode=4)
    assert torch.equal(r3["f64"], r4["f64"]) and torch.equal(r3["g64"], r4["g64"])
    h5 = fs.fs_sinkhorn_dense_ex(geo["C"], a, b, w.eps, 20, 0.0, kernel_mode=4)
    res5 = h5.result()
    assert res5["iters"] == 20 and torch.equal(h5.f, r3["f"]) and torch.equal(h5.g, r3["g"])
    # max_iter = 0 returns the start
    r0 = fs.fs_sinkhorn_solve(a, b, w.eps, 0, 0.0, C=geo["C"], kernel_mode=4)
    assert r0["iters"] == 0 and float(r0["f"].abs().max()) == 0.0 and float(r0["g"].abs().max()) == 0.0
    # shapes it does not take
    with pytest.raises(fs.FsError, match="kernel_mode 4"):
        fs.fs_sinkhorn_solve(a, torch.full((1025,), 1 / 1025, device="cuda"), w.eps, 3, 0.0,
                             C=torch.zeros(300, 1025, device="cuda"), kernel_mode=4)
    u = torch.full((1024,), 1 / 1024, device="cuda")
    with pytest.raises(fs.FsError, match="kernel_mode 4"):
        fs.fs_sinkhorn_solve(u, u, w.eps, 3, 0.0, X=torch.zeros(1024, 3, device="cuda"),
                             Y=torch.zeros(1024, 3, device="cuda"), kernel_mode=4)


# ------------------------------------------------------------------ one launch over the whole chip (n, m <= 4096)
def _needs_whole_chip():
    """The shapes below assume the 256 compute units of an unpartitioned MI355X (one workgroup each)."""
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    if cus < 256:
        pytest.skip(f"kernel_mode 5 shapes of this test need 256 compute units, the device has {cus}")


@pytest.mark.parametrize("n,m,iters", [(1, 1, 20), (5, 7, 20), (257, 300, 20), (1024, 1024, 12), (1000, 2048, 12),
                                       (300, 2000, 12), (4000, 300, 12), (2048, 2048, 8), (4096, 1024, 8),
                                       (3000, 777, 8), (1500, 1025, 8)])
def test_grid_kernel_matches_oracle(fs, oracle, n, m, iters):
    """kernel_mode = 5: the whole solve in one launch over up to 256 workgroups, C in registers, two grid-wide
    waits per iteration."""
    _needs_whole_chip()
    w = W.random_dense(n, m, seed=7900 + n + m, cmax=2.0, eps=0.02)
    if n > 8:
        w.a[2::9] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, iters, kernel_mode=5)
    assert e64 < TOL_F64 and e32 < TOL_F32, (e64, e32)
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


@pytest.mark.parametrize("n,m,d", [(5, 7, 2), (1000, 1200, 3), (2048, 1024, 2), (700, 300, 17), (300, 2000, 3),
                                   (1500, 900, 64)])
def test_grid_kernel_point_clouds(fs, oracle, n, m, d):
    """kernel_mode = 5 on point clouds: squared distances formed once in fp64 and kept in registers."""
    _needs_whole_chip()
    w = W.random_points(n, m, d, seed=7980 + n + m + d, eps=0.02)
    if n > 8:
        w.a[2::9] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    r, ref, e64, e32 = _solve_and_compare(fs, oracle, w, 15, kernel_mode=5)
    assert e64 < TOL_F64 and e32 < TOL_F32, (e64, e32)
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], X=w.X, Y=w.Y))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7
    r1, _, _, _ = _solve_and_compare(fs, oracle, w, 15, kernel_mode=1)       # the multi-kernel point-cloud path
    assert float((r1["f64"] - r["f64"]).abs().max()) / w.eps < TOL_F64


def test_grid_kernel_stop_rule_history_and_resume(fs, oracle):
    _needs_whole_chip()
    import torch
    w = W.random_dense(600, 1300, seed=7950, cmax=1.0, eps=0.05)
    geo, a, b = to_dev(w)
    ref = oracle.solve(w.a, w.b, w.eps, 400, tol=1e-5, check_every=7, C=w.C, err_every_iter=True)
    hist = torch.full((400,), float("nan"), dtype=torch.float32, device="cuda")
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 400, 1e-5, C=geo["C"], want_f64=True, check_every=7, kernel_mode=5,
                             err_history=hist)
    assert r["converged"] and ref["converged"]
    assert abs(r["iters"] - int(ref["iters"])) <= 7 and r["iters"] % 7 == 0
    k = r["iters"]
    refk = oracle.solve(w.a, w.b, w.eps, k, C=w.C)
    assert pot_err(r["f64"].cpu().numpy(), refk["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), refk["g"], w.eps) < TOL_F64
    h = hist.cpu().numpy()
    eh = np.asarray(ref["err_hist"], dtype=np.float64)
    upto = min(k, int(ref["iters"]))
    assert np.all(np.isfinite(h[:upto]))
    assert np.allclose(h[:upto], eh[:upto], rtol=2e-3, atol=5e-7)
    assert np.all(np.isnan(h[k:]))
    rm = fs.fs_sinkhorn_solve(a, b, w.eps, 400, 1e-5, C=geo["C"], want_f64=True, check_every=7, kernel_mode=1)
    assert rm["iters"] == k and float((rm["f64"] - r["f64"]).abs().max()) / w.eps < TOL_F64
    # fixed count without the trailing error pass; resume from fp64 potentials = one longer run
    r1 = fs.fs_sinkhorn_solve(a, b, w.eps, 11, 0.0, C=geo["C"], want_f64=True, kernel_mode=5, skip_final_err=True)
    assert math.isnan(r1["marginal_err"]) and r1["iters"] == 11
    r2 = fs.fs_sinkhorn_solve(a, b, w.eps, 9, 0.0, C=geo["C"], want_f64=True, kernel_mode=5, warm_start=True,
                              f64_in=r1["f64"], g64_in=r1["g64"])
    r3 = fs.fs_sinkhorn_solve(a, b, w.eps, 20, 0.0, C=geo["C"], want_f64=True, kernel_mode=5)
    assert float((r2["f64"] - r3["f64"]).abs().max()) / w.eps < 1e-9
    assert float((r2["g64"] - r3["g64"]).abs().max()) / w.eps < 1e-9
    r4 = fs.fs_sinkhorn_solve(a, b, w.eps, 20, 0.0, C=geo["C"], want_f64=True, kernel_mode=5)
    assert torch.equal(r3["f64"], r4["f64"]) and torch.equal(r3["g64"], r4["g64"])
    h5 = fs.fs_sinkhorn_dense_ex(geo["C"], a, b, w.eps, 20, 0.0, kernel_mode=5)
    res5 = h5.result()
    assert res5["iters"] == 20 and torch.equal(h5.f, r3["f"]) and torch.equal(h5.g, r3["g"])
    r0 = fs.fs_sinkhorn_solve(a, b, w.eps, 0, 0.0, C=geo["C"], kernel_mode=5)
    assert r0["iters"] == 0 and float(r0["f"].abs().max()) == 0.0 and float(r0["g"].abs().max()) == 0.0
    # a forced give-up is clean, and the next solve is unaffected
    rg = fs.fs_sinkhorn_solve(a, b, w.eps, 30, 0.0, C=geo["C"], kernel_mode=5, wait_limit=1)
    assert rg["nonfinite"] or rg["iters"] == 30
    r6 = fs.fs_sinkhorn_solve(a, b, w.eps, 20, 0.0, C=geo["C"], want_f64=True, kernel_mode=5)
    assert torch.equal(r3["f64"], r6["f64"])
    # shapes it does not take: too few rows for that many columns, too many entries per lane
    u16 = torch.full((16,), 1 / 16, device="cuda")
    with pytest.raises(fs.FsError, match="kernel_mode 5"):
        fs.fs_sinkhorn_solve(u16, torch.full((2048,), 1 / 2048, device="cuda"), w.eps, 3, 0.0,
                             C=torch.zeros(16, 2048, device="cuda"), kernel_mode=5)
    u4k = torch.full((4096,), 1 / 4096, device="cuda")
    with pytest.raises(fs.FsError, match="kernel_mode 5"):
        fs.fs_sinkhorn_solve(u4k, torch.full((2048,), 1 / 2048, device="cuda"), w.eps, 3, 0.0,
                             C=torch.zeros(4096, 2048, device="cuda"), kernel_mode=5)


@pytest.mark.parametrize("n,m,warm", [(300, 410, False), (1000, 1200, False), (900, 1100, True)])
def test_one_launch_solvers_fall_back_when_they_give_up(fs, oracle, n, m, warm):
    """Automatic mode with wait_limit = 1: the library's own choice of a one-launch kernel almost surely gives
    up on its first wait; the blocking solve must then deliver the right answer through the multi-kernel driver,
    also when the starting potentials were passed in place."""
    import torch
    w = W.random_dense(n, m, seed=8100 + n, cmax=1.0, eps=0.05)
    geo, a, b = to_dev(w)
    kw = {}
    f0 = g0 = None
    if warm:
        rng = np.random.default_rng(5)
        f0 = (rng.standard_normal(n) * 0.1).astype(np.float32)
        g0 = (rng.standard_normal(m) * 0.1).astype(np.float32)
        kw = dict(f=dev(f0), g=dev(g0), warm_start=True)
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 25, 0.0, C=geo["C"], want_f64=True, wait_limit=1, **kw)
    ref = oracle.solve(w.a, w.b, w.eps, 25, C=w.C, f0=f0, g0=g0) if warm else oracle.solve(w.a, w.b, w.eps, 25, C=w.C)
    assert r["iters"] == 25 and not r["nonfinite"] and not r["gave_up"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    # asked for by name, the same kernel reports that it gave up (or, with luck, finishes)
    if n * m > 1 << 18:
        _needs_whole_chip()
    rk = fs.fs_sinkhorn_solve(a, b, w.eps, 25, 0.0, C=geo["C"], kernel_mode=4 if n * m <= 1 << 18 else 5, wait_limit=1)
    assert rk["gave_up"] or (rk["iters"] == 25 and not rk["nonfinite"])


def test_coop_kernel_bounded_wait_gives_up_cleanly(fs, oracle):
    """wait_limit = 1: a workgroup stops waiting for the others after a single poll.  Whether that is enough
    depends on timing, so either outcome is legal - but nothing in between: the solve is either complete and
    right, or it says so (nonfinite = 1, no error value, not converged).  Every workgroup exits either way, and the next
    solve on the same workspace is unaffected."""
    import torch
    w = W.random_dense(512, 500, seed=7700, cmax=1.0, eps=0.05)
    geo, a, b = to_dev(w)
    ref = oracle.solve(w.a, w.b, w.eps, 30, C=w.C)
    outcomes = set()
    for _ in range(6):
        r = fs.fs_sinkhorn_solve(a, b, w.eps, 30, 0.0, C=geo["C"], want_f64=True, kernel_mode=4, wait_limit=1)
        if r["nonfinite"]:
            outcomes.add("gave up")          # potentials are then not valid (NaN where a workgroup had stopped)
            assert math.isnan(r["marginal_err"]) and not r["converged"] and 0 <= r["iters"] <= 30
        else:
            outcomes.add("completed")
            assert r["iters"] == 30 and pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 30, 0.0, C=geo["C"], want_f64=True, kernel_mode=4)
    assert r["iters"] == 30 and not r["nonfinite"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    print("outcomes with wait_limit = 1:", sorted(outcomes))


@pytest.mark.parametrize("B,n,m", [(1, 64, 64), (7, 100, 90), (300, 64, 64), (33, 256, 256)])
def test_batched_small_solves(fs, oracle, B, n, m):
    import torch
    ws = [W.random_dense(n, m, seed=7200 + 13 * q + n, cmax=1.5, eps=0.03) for q in range(B)]
    C = torch.from_numpy(np.stack([w.C for w in ws])).cuda()
    a = torch.from_numpy(np.stack([w.a for w in ws])).cuda()
    b = torch.from_numpy(np.stack([w.b for w in ws])).cuda()
    out = fs.fs_sinkhorn_dense_batched(C, a, b, ws[0].eps, 30, 0.0, want_f64=True)
    res = fs.results_from_device(out["result"])
    f64, g64 = out["f64"].cpu().numpy(), out["g64"].cpu().numpy()
    for q in sorted(set([0, B // 2, B - 1] + list(range(0, B, max(1, B // 6))))):
        ref = oracle.solve(ws[q].a, ws[q].b, ws[q].eps, 30, C=ws[q].C)
        assert res[q]["iters"] == 30 and not res[q]["nonfinite"]
        assert pot_err(f64[q], ref["f"], ws[q].eps) < TOL_F64 and pot_err(g64[q], ref["g"], ws[q].eps) < TOL_F64
        err_ref = float(oracle.marginal_err(ws[q].a, ws[q].b, ws[q].eps, ref["f"], ref["g"], C=ws[q].C))
        assert abs(res[q]["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7
    # problems stop independently: a tolerance only the easy ones reach
    out2 = fs.fs_sinkhorn_dense_batched(C, a, b, ws[0].eps, 500, 1e-4, check_every=5)
    res2 = fs.results_from_device(out2["result"])
    ref0 = oracle.solve(ws[0].a, ws[0].b, ws[0].eps, 500, tol=1e-4, check_every=5, C=ws[0].C)
    assert res2[0]["converged"] == bool(ref0["converged"]) and abs(res2[0]["iters"] - int(ref0["iters"])) <= 5
    with pytest.raises(fs.FsError):
        fs.fs_sinkhorn_dense_batched(torch.zeros((2, 300, 8), device="cuda"), torch.ones((2, 300), device="cuda"),
                                     torch.ones((2, 8), device="cuda"), 0.1, 3, 0.0)


# ------------------------------------------------------------------ stopping rule, history, resume
@pytest.mark.parametrize("kind,mode", [("dense", 1), ("dense", 2), ("points", 0)])
def test_stopping_rule_and_history(fs, oracle, kind, mode):
    import torch
    w = W.random_dense(96, 128, seed=9, eps=0.05) if kind == "dense" else W.random_points(96, 120, 3, seed=9, eps=0.05)
    geo, a, b = to_dev(w)
    tol, K = 1e-5, 400        # well above the ~1e-7 fp32 noise floor of the device-side error
    full = oracle.solve(w.a, w.b, w.eps, K, C=w.C, X=w.X, Y=w.Y, err_every_iter=True)
    eh = full["err_hist"]
    for c in (1, 7, 10):
        hist = torch.full((K,), float("nan"), dtype=torch.float32, device="cuda")
        r = fs.fs_sinkhorn_solve(a, b, w.eps, K, tol, want_f64=True, check_every=c, kernel_mode=mode,
                                 err_history=hist, **geo)
        ks = [k for k in range(c, K + 1, c) if eh[k - 1] < tol]
        assert r["converged"] and r["iters"] == ks[0]
        ref = oracle.solve(w.a, w.b, w.eps, r["iters"], C=w.C, X=w.X, Y=w.Y)
        assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
        assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
        assert abs(r["marginal_err"] - eh[r["iters"] - 1]) <= 1e-3 * eh[r["iters"] - 1] + 5e-7
        h = hist.cpu().numpy()[:r["iters"]]
        assert np.all(np.isfinite(h))
        assert np.allclose(h, eh[:r["iters"]], rtol=1e-3, atol=5e-7)
    # not reached: runs to max_iter, reports not converged, err of the last iterate
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 15, 1e-30, check_every=5, kernel_mode=mode, **geo)
    assert r["iters"] == 15 and not r["converged"]
    assert abs(r["marginal_err"] - eh[14]) <= 1e-3 * eh[14] + 5e-7
    # max_iter = 0 returns the start
    r0 = fs.fs_sinkhorn_solve(a, b, w.eps, 0, 0.0, kernel_mode=mode, **geo)
    assert r0["iters"] == 0 and float(r0["f"].abs().max()) == 0.0 and float(r0["g"].abs().max()) == 0.0


@pytest.mark.parametrize("kind,mode", [("dense", 1), ("dense", 2), ("points", 0)])
def test_warm_start_resume_and_determinism(fs, kind, mode):
    import torch
    w = W.random_dense(80, 256, seed=19, eps=0.05) if kind == "dense" else W.random_points(80, 250, 3, seed=19, eps=0.05)
    geo, a, b = to_dev(w)
    r1 = fs.fs_sinkhorn_solve(a, b, w.eps, 13, 0.0, want_f64=True, kernel_mode=mode, **geo)
    r2 = fs.fs_sinkhorn_solve(a, b, w.eps, 9, 0.0, want_f64=True, kernel_mode=mode, warm_start=True,
                              f64_in=r1["f64"], g64_in=r1["g64"], **geo)
    r3 = fs.fs_sinkhorn_solve(a, b, w.eps, 22, 0.0, want_f64=True, kernel_mode=mode, **geo)
    # not bitwise: the hand-over multiplies and divides by log2(e)/eps once, and the fused kernel walks
    # the row panels in an order that depends on the parity of the iteration counter, which restarts
    # at 0 on resume (a different fp32 summation order).  Equal to fp32-sum noise.
    assert float((r2["f64"] - r3["f64"]).abs().max()) / w.eps < TOL_F64
    assert float((r2["g64"] - r3["g64"]).abs().max()) / w.eps < TOL_F64
    # run-to-run determinism: no result depends on the order in which workgroups finish
    r4 = fs.fs_sinkhorn_solve(a, b, w.eps, 22, 0.0, want_f64=True, kernel_mode=mode, **geo)
    assert torch.equal(r4["f64"], r3["f64"]) and torch.equal(r4["g"], r3["g"])


@pytest.mark.parametrize("kind,mode", [("dense", 1), ("dense", 2), ("points", 0)])
def test_graph_replayed_blocks_match_plain_launches(fs, kind, mode):
    """Blocks of check_every iterations replayed as one hipGraph: several solves in a row, eager work and
    synchronisations between them, fixed-count and stop-by-tolerance; every one must equal the
    plain-launch result bit for bit."""
    import torch
    w = W.random_dense(96, 256, seed=29, eps=0.05) if kind == "dense" else W.random_points(96, 250, 3, seed=29, eps=0.05)
    geo, a, b = to_dev(w)
    for max_iter, tol in ((37, 0.0), (400, 1e-5), (60, 0.0)):
        ref = fs.fs_sinkhorn_solve(a, b, w.eps, max_iter, tol, want_f64=True, kernel_mode=mode, use_graph=1, **geo)
        for rep in range(3):
            junk = (torch.rand(1000, device="cuda") * 2).sum()       # unrelated eager work between replays
            r = fs.fs_sinkhorn_solve(a, b, w.eps, max_iter, tol, want_f64=True, kernel_mode=mode, use_graph=2, **geo)
            torch.cuda.synchronize()
            assert r["iters"] == ref["iters"] and r["converged"] == ref["converged"]
            assert torch.equal(r["f64"], ref["f64"]) and torch.equal(r["g64"], ref["g64"])
            assert r["marginal_err"] == ref["marginal_err"] or (math.isnan(r["marginal_err"]) and math.isnan(ref["marginal_err"]))
            assert float(junk) > 0


@pytest.mark.parametrize("kind,mode", [("dense", 2), ("dense", 4), ("dense_small", 3), ("points", 0), ("points_small", 4)])
def test_async_entry_points_replay_from_a_captured_graph(fs, kind, mode):
    """The asynchronous entry points only enqueue kernels (no host synchronisation, no memset nodes), so a caller
    may capture them into a graph of its own.  Each replay - with eager solves and synchronisations in between -
    must reproduce the eager result bit for bit."""
    import torch
    if kind == "dense":
        w = W.random_dense(300, 1100 if mode == 2 else 700, seed=8800 + mode, cmax=2.0, eps=0.03)
    elif kind == "dense_small":
        w = W.random_dense(100, 120, seed=8810, cmax=2.0, eps=0.03)
    elif kind == "points":
        w = W.random_points(900, 1300, 3, seed=8820, eps=0.03)
    else:
        w = W.random_points(200, 260, 3, seed=8830, eps=0.03)
    geo, a, b = to_dev(w)
    dense = w.C is not None
    d = 0 if dense else 3
    f = torch.empty(w.n, dtype=torch.float32, device="cuda")
    g = torch.empty(w.m, dtype=torch.float32, device="cuda")
    ws = torch.empty(fs.fs_workspace_bytes(w.n, w.m, d), dtype=torch.uint8, device="cuda")

    def enqueue():
        if dense:
            return fs.fs_sinkhorn_dense_ex(geo["C"], a, b, w.eps, 30, 0.0, f=f, g=g, workspace=ws, kernel_mode=mode)
        return fs.fs_sinkhorn_points_ex(geo["X"], geo["Y"], a, b, w.eps, 30, 0.0, f=f, g=g, workspace=ws, kernel_mode=mode)

    h = enqueue()
    assert h.result()["iters"] == 30
    f_ref, g_ref = f.clone(), g.clone()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        hg = enqueue()
    other = W.random_dense(130, 90, seed=8899, cmax=1.0, eps=0.05)
    for rep in range(3):
        f.fill_(float("nan"))
        g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(f, f_ref) and torch.equal(g, g_ref), rep
        assert hg.result()["iters"] == 30
        # eager work of the library between the replays
        fs.fs_sinkhorn_solve(dev(other.a), dev(other.b), other.eps, 7, 0.0, C=dev(other.C))
        torch.cuda.synchronize()


def test_blocking_and_async_entry_points_agree(fs):
    import torch
    w = W.random_dense(200, 512, seed=23, eps=0.05)
    geo, a, b = to_dev(w)
    f1, g1, it1 = fs.fs_sinkhorn_dense(geo["C"], a, b, w.eps, 300, 1e-6)
    h = fs.fs_sinkhorn_dense_ex(geo["C"], a, b, w.eps, 300, 1e-6)
    res = h.result()
    assert res["iters"] == it1 and res["converged"]
    assert torch.equal(h.f, f1) and torch.equal(h.g, g1)
    wp = W.random_points(150, 170, 3, seed=24, eps=0.05)
    geop, ap, bp = to_dev(wp)
    f2, g2, it2 = fs.fs_sinkhorn_points(geop["X"], geop["Y"], ap, bp, wp.eps, 300, 1e-6)
    hp = fs.fs_sinkhorn_points_ex(geop["X"], geop["Y"], ap, bp, wp.eps, 300, 1e-6)
    resp = hp.result()
    assert resp["iters"] == it2 and torch.equal(hp.f, f2) and torch.equal(hp.g, g2)
    assert it2 % 10 == 0 and it1 % 10 == 0          # default check interval c = 10


# ------------------------------------------------------------------ plan and cost
@pytest.mark.parametrize("kind", ["dense", "dense_odd", "points", "points1", "points6", "points20", "points64"])
def test_plan_and_cost(fs, oracle, kind):
    if kind == "dense":
        w = W.random_dense(130, 300, seed=31, eps=0.04)
    elif kind == "dense_odd":
        w = W.random_dense(77, 4099, seed=33, eps=0.04)
    else:
        d = int(kind[6:] or 3)
        w = W.random_points(130 + 7 * d, 257 + d, d, seed=31 + d, eps=0.04)
        w.b[4] = 0.0
        w.b[:] = w.b / w.b.sum(dtype=np.float64)
    geo, a, b = to_dev(w)
    ref = oracle.solve(w.a, w.b, w.eps, 40, C=w.C, X=w.X, Y=w.Y)
    f32, g32 = ref["f"].astype(np.float32), ref["g"].astype(np.float32)
    P = fs.fs_plan(a, b, w.eps, dev(f32), dev(g32), **geo).cpu().numpy().astype(np.float64)
    P_ref = oracle.plan(w.a, w.b, w.eps, f32.astype(np.float64), g32.astype(np.float64), C=w.C, X=w.X, Y=w.Y)
    assert np.max(np.abs(P - P_ref) / (P_ref + 1e-30 + 1e-6 * P_ref.max())) < 2e-5
    c = float(fs.fs_cost(a, b, w.eps, dev(f32), dev(g32), **geo).cpu()[0])
    c_ref = float(oracle.cost(w.a, w.b, w.eps, f32.astype(np.float64), g32.astype(np.float64), C=w.C, X=w.X, Y=w.Y))
    assert abs(c - c_ref) <= 1e-5 * abs(c_ref)
    P64 = fs.fs_plan(a, b, w.eps, dev(ref["f"]), dev(ref["g"]), **geo).cpu().numpy().astype(np.float64)
    P64_ref = oracle.plan(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C, X=w.X, Y=w.Y)
    assert np.max(np.abs(P64 - P64_ref) / (P64_ref + 1e-30 + 1e-6 * P64_ref.max())) < 2e-5
    c64 = float(fs.fs_cost(a, b, w.eps, dev(ref["f"]), dev(ref["g"]), **geo).cpu()[0])
    assert abs(c64 - float(oracle.cost(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C, X=w.X, Y=w.Y))) <= 1e-5 * abs(c_ref)


# ------------------------------------------------------------------ closed form at size (independent of the oracle)
@pytest.mark.parametrize("kind,n,m,d", [("dense", 300, 257, 0), ("dense", 130, 4100, 0), ("dense", 1000, 8192, 0),
                                         ("dense", 33, 1, 0), ("dense", 90, 4101, 0), ("dense", 50, 6, 0),
                                         ("points", 700, 1300, 3), ("points", 1030, 500, 2),
                                         ("points", 90, 200, 7), ("points", 300, 1000, 16), ("points", 520, 130, 33),
                                         ("points", 129, 257, 64),
                                         # small problems: one single-workgroup launch
                                         ("dense", 100, 120, 0), ("dense", 1, 1, 0), ("dense", 5, 1000, 0),
                                         ("points", 200, 210, 3), ("points", 31, 64, 1), ("points", 256, 255, 4),
                                         ("points", 8300, 150, 3), ("points", 150, 8300, 2), ("points", 2100, 1990, 1)])
@pytest.mark.parametrize("precision", ["f32", "f64"])
def test_diagnostics_one_pass(fs, oracle, kind, n, m, d, precision):
    """fs_diagnostics against the oracle's direct definitions (explicit plan, own sums): cost, mass, KL,
    primal, dual, both marginals and their L1 errors, from potentials that are NOT converged (so that
    no term vanishes) and with some zero weights."""
    w = W.random_dense(n, m, seed=6000 + n + m, cmax=2.0, eps=0.05) if kind == "dense" else \
        W.random_points(n, m, d, seed=6000 + n + m + d, eps=0.05)
    if n > 40:
        w.a[5::11] = 0.0
        w.a[:] = w.a / w.a.sum(dtype=np.float64)
    if m > 40:                                  # zero column weights too: plan columns of exact zeros
        w.b[3::13] = 0.0
        w.b[:] = w.b / w.b.sum(dtype=np.float64)
    ref = oracle.solve(w.a, w.b, w.eps, 3, C=w.C, X=w.X, Y=w.Y)
    f_h, g_h = ref["f"], ref["g"]
    if precision == "f32":
        f_h, g_h = f_h.astype(np.float32).astype(np.float64), g_h.astype(np.float32).astype(np.float64)
    import torch
    geo, a, b = to_dev(w)
    dt = torch.float32 if precision == "f32" else torch.float64
    r = fs.fs_diagnostics(a, b, w.eps, dev(f_h, dt), dev(g_h, dt), want_marginals=True, **geo)
    out = r["out"].cpu().numpy()
    o = oracle.objectives(w.a, w.b, w.eps, f_h, g_h, C=w.C, X=w.X, Y=w.Y)
    ro, co = oracle.marginals(w.a, w.b, w.eps, f_h, g_h, C=w.C, X=w.X, Y=w.Y)
    got = dict(zip(fs.DIAG_FIELDS, out))
    for key in ("cost", "mass", "kl", "primal", "dual"):
        assert abs(got[key] - float(o[key])) <= 2e-6 * max(1.0, abs(float(o[key]))), (key, got[key], float(o[key]))
    assert np.abs(r["row_marginal"].cpu().numpy() - ro).sum() <= 2e-6
    assert np.abs(r["col_marginal"].cpu().numpy() - co).sum() <= 2e-6
    assert abs(got["row_err"] - np.abs(ro - w.a).sum()) <= 2e-6
    assert abs(got["col_err"] - np.abs(co - w.b).sum()) <= 2e-6
    # the stand-alone cost entry point agrees
    cost2 = float(fs.fs_cost(a, b, w.eps, dev(f_h, dt), dev(g_h, dt), **geo).cpu()[0])
    assert abs(cost2 - got["cost"]) <= 2e-6 * max(1.0, abs(got["cost"]))


@pytest.mark.parametrize("kind,n,m,d,dz", [("dense", 300, 257, 0, 3), ("dense", 130, 4100, 0, 1), ("dense", 700, 8192, 0, 4),
                                            ("dense", 17, 3, 0, 2), ("dense", 61, 4102, 0, 3), ("dense", 1000, 1024, 0, 2), ("dense", 129, 2052, 0, 4),
                                            ("dense", 5000, 1028, 0, 3), ("points", 700, 1300, 3, 3), ("points", 1030, 500, 2, 4),
                                            ("points", 90, 200, 7, 2), ("points", 400, 300, 12, 4), ("points", 131, 1025, 40, 1),
                                            ("points", 260, 64, 64, 3), ("points", 8300, 140, 3, 2),
                                            ("points", 2100, 1990, 4, 3)])
def test_barycentric_mapping(fs, oracle, kind, n, m, d, dz):
    """fs_barycentric against the oracle's explicit-plan definition; a zero-weight row maps to 0."""
    import torch
    w = W.random_dense(n, m, seed=6500 + n + m, cmax=2.0, eps=0.05) if kind == "dense" else \
        W.random_points(n, m, d, seed=6500 + n + m + d, eps=0.05)
    w.a[1] = 0.0
    w.a[:] = w.a / w.a.sum(dtype=np.float64)
    if m > 8:
        w.b[2::7] = 0.0                         # targets without mass take no part in the mapping
        w.b[:] = w.b / w.b.sum(dtype=np.float64)
    ref = oracle.solve(w.a, w.b, w.eps, 4, C=w.C, X=w.X, Y=w.Y)
    rng = np.random.default_rng(n + m)
    Z = rng.standard_normal((m, dz)).astype(np.float32) if kind == "dense" or dz != d else w.Y.copy()
    geo, a, b = to_dev(w)
    To = oracle.barycentric(w.a, w.b, w.eps, ref["f"], ref["g"], Z.astype(np.float64), C=w.C, X=w.X, Y=w.Y)
    scale = 1.0 + float(np.abs(Z).max())
    for dt in (torch.float64, torch.float32):
        f_h = ref["f"] if dt == torch.float64 else ref["f"].astype(np.float32).astype(np.float64)
        g_h = ref["g"] if dt == torch.float64 else ref["g"].astype(np.float32).astype(np.float64)
        To_dt = To if dt == torch.float64 else oracle.barycentric(w.a, w.b, w.eps, f_h, g_h, Z.astype(np.float64),
                                                                   C=w.C, X=w.X, Y=w.Y)
        T = fs.fs_barycentric(a, b, w.eps, dev(f_h, dt), dev(g_h, dt), dev(Z), **geo).cpu().numpy()
        assert T.shape == (n, dz)
        assert np.abs(T - To_dt).max() <= 5e-6 * scale, float(np.abs(T - To_dt).max())
        assert np.all(T[1] == 0.0)
    with pytest.raises(fs.FsError):
        fs.fs_barycentric(a, b, w.eps, dev(ref["f"], torch.float64), dev(ref["g"], torch.float64),
                          torch.zeros((m, 5), device="cuda"), **geo)


@pytest.mark.parametrize("mode", [1, 2])
def test_separable_cost_closed_form_large(fs, mode):
    """C_ij = u_i + v_j (exactly representable) => after ONE iteration f = u + kappa, g = v - kappa - eps log(sum a),
    and every later iteration is a fixed point of the plan (err = |sum a - sum b| only)."""
    import torch
    n, m, eps = 2048, 4096, float(np.float32(0.01))
    rng = np.random.default_rng(5)
    u = (rng.integers(0, 1024, n) / 256.0)
    v = (rng.integers(0, 1024, m) / 256.0)
    C = (u[:, None] + v[None, :]).astype(np.float32)
    assert np.array_equal(C.astype(np.float64), u[:, None] + v[None, :])
    w = W.random_dense(8, 8, seed=1)
    a = W._dirichlet(rng, n, 1.0)
    b = W._dirichlet(rng, m, 1.0)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    r = fs.fs_sinkhorn_solve(dev(a), dev(b), eps, 1, 0.0, C=dev(C), want_f64=True, kernel_mode=mode)
    vm = (-v / eps).max()
    kappa = -eps * (vm + np.log(np.sum(b64 * np.exp(-v / eps - vm))))
    f_ref = u + kappa
    g_ref = v - kappa - eps * np.log(a64.sum())
    assert pot_err(r["f64"].cpu().numpy(), f_ref, eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), g_ref, eps) < TOL_F64
    assert r["marginal_err"] < 1e-6
    r5 = fs.fs_sinkhorn_solve(dev(a), dev(b), eps, 5, 0.0, C=dev(C), want_f64=True, kernel_mode=mode)
    fsum = (r5["f64"].cpu().numpy()[:, None] + r5["g64"].cpu().numpy()[None, :] - C.astype(np.float64))
    assert np.ptp(fsum) / eps < 1e-4          # f_i + g_j - C_ij is one constant: P = a x b up to normalisation


# ------------------------------------------------------------------ degenerate inputs and argument errors
def test_zero_weights_and_singletons(fs, oracle):
    w = W.random_dense(40, 64, seed=41, eps=0.05)
    a = w.a.copy(); a[7] = 0.0
    b = w.b.copy(); b[11] = 0.0
    for mode in (1, 2):
        r = fs.fs_sinkhorn_solve(dev(a), dev(b), w.eps, 30, 0.0, C=dev(w.C), want_f64=True, kernel_mode=mode)
        ref = oracle.solve(a, b, w.eps, 30, C=w.C)
        assert not r["nonfinite"]
        assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
        assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    one = np.ones(1, dtype=np.float32)
    C11 = np.array([[0.7]], dtype=np.float32)
    r = fs.fs_sinkhorn_solve(dev(one), dev(one), 0.1, 3, 0.0, C=dev(C11), want_f64=True)
    ref = oracle.solve(one, one, float(np.float32(0.1)), 3, C=C11)
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], 0.1) < TOL_F64


def test_zero_weights_on_the_prefetch_fused_path(fs, oracle):
    """m in (4096, 8192] runs the LDS-prefetch fused kernel; a zero column weight makes that column's
    FAST-mode partial undefined, which the combine kernel must notice and recompute."""
    w = W.random_dense(48, 8192, seed=45, eps=0.05)
    a = w.a.copy(); a[7] = 0.0
    b = w.b.copy(); b[11] = 0.0; b[5000] = 0.0
    r = fs.fs_sinkhorn_solve(dev(a), dev(b), w.eps, 30, 0.0, C=dev(w.C), want_f64=True, kernel_mode=2)
    ref = oracle.solve(a, b, w.eps, 30, C=w.C)
    assert not r["nonfinite"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64


def test_nonfinite_cost_is_flagged_not_fatal(fs):
    w = W.random_dense(32, 64, seed=43, eps=0.05)
    C = w.C.copy(); C[3, 5] = np.nan
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, 5, 1e-9, C=dev(C), kernel_mode=1)
    assert r["nonfinite"] and r["iters"] == 5 and not r["converged"]


def test_argument_errors(fs):
    import torch
    w = W.random_dense(8, 8, seed=2)
    geo, a, b = to_dev(w)
    C = geo["C"]
    for kw in (dict(eps=0.0), dict(eps=-1.0), dict(eps=float("nan")), dict(eps=float("inf")), dict(max_iter=-1)):
        args = dict(eps=w.eps, max_iter=3)
        args.update(kw)
        with pytest.raises(fs.FsError) as e:
            fs.fs_sinkhorn_dense(C, a, b, args["eps"], args["max_iter"], 0.0)
        assert e.value.status == fs.FS_ERR_INVALID_ARG and fs.fs_last_error()
    X = torch.zeros((8, 65), device="cuda")
    with pytest.raises(fs.FsError) as e:
        fs.fs_sinkhorn_points(X, X, a, b, 0.1, 3, 0.0)
    assert e.value.status == fs.FS_ERR_INVALID_ARG
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(fs.FsError) as e:
        fs.fs_sinkhorn_dense_ex(C, a, b, w.eps, 3, 0.0, workspace=small)
    assert e.value.status == fs.FS_ERR_WORKSPACE
