"""GPU parity of the persistent fused pass (kernel_mode 6; the automatic choice of the blocking dense
solves for 128 < m <= 8192): one resident workgroup per compute unit, a block of iterations per launch,
two grid-wide waits per iteration.  Everything goes through the C ABI and is compared with the CPU oracle.
"""
import math

import numpy as np
import pytest

from paper_2605_00837_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_F32, TOL_F64 = 1e-3, 2e-5


@pytest.fixture(scope="module")
def fs():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_00837_amd import binding
    return binding


def dev(x):
    import torch
    return None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _supported(fs, n, m):
    """The kernel needs one workgroup per strip of at most 64 columns: enough row panels and compute units."""
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    try:
        return fs.fs_kernel_choice(n, m, 0, True, cus, kernel_mode=6) == "persist"
    except fs.FsError:
        return False


def pot_err(x, ref, eps):
    return float(np.max(np.abs(np.asarray(x, dtype=np.float64) - ref)) / eps)


# every instantiation: one to four 16-byte groups per lane, full and masked widths; ragged last panels; many
# panels per workgroup; grids smaller than the chip; strips that are not a power of two wide
SHAPES = [(255, 8192), (300, 8190), (517, 4100), (2049, 4096), (300, 1100), (1000, 16001), (333, 12288), (260, 16384),
          (70, 2000), (3001, 5000), (129, 4096), (200, 1028), (1100, 6001), (600, 9000),
          (4099, 4096), (2047, 4096), (9001, 4096),      # 4096 columns: panels of 4 rows from 2048 rows up, of 2 below
          (4096, 4096), (1024, 4096), (3070, 4096), (2048, 8192), (1500, 8192),   # shares of C that stay on the chip
          (2100, 8192), (6001, 4096), (12000, 4096), (13000, 4096), (6200, 8192), (17000, 4096), (8300, 8192),
          (3000, 3000), (1500, 2049), (4000, 4095), (2000, 6145), (1025, 8191), (1200, 5000), (1023, 4097),   # ... idle lanes
          (2048, 2048), (8190, 2048), (3000, 1500), (5000, 1025), (2051, 2047), (20000, 2048), (70000, 2048),   # panels of 8 rows
          (4200, 2500), (8300, 1500), (2200, 5000), (2300, 8000), (6000, 6000), (9000, 3000), (5000, 6145),
          (2048, 6144), (5000, 6144), (1000, 6000), (2301, 4097),   # ... and shares of which the 512-lane kernel streams a part
          (1000, 1000), (4096, 1024), (8191, 1024), (333, 700), (5000, 513), (9000, 1024),   # two row groups per workgroup
          (17000, 1024), (20000, 1000), (4700, 8100), (9300, 8192),    # ... streamed
          (22000, 4096), (11500, 7000),                            # ... 22 / 23 panels per workgroup (masked: the 512-lane kernel on request only)
          (2100, 512), (8190, 512), (1000, 300), (4097, 257), (33000, 512), (40000, 400),   # four row groups; streamed
          (5000, 256), (4500, 129), (16383, 256), (70000, 256), (66000, 200)]                 # eight row groups; streamed


def _resident(n, m, cus=256, most=4):
    """Whether the 512-lane kernel of the persistent pass takes the shape (128 < m <= 8192, 1 .. most panels of 64 KiB
    per workgroup of a grid of min(cus, panels) workgroups that merge at most 64 columns each): up to 4 panels the matrix stays on the chip for a whole launch; beyond
    that the panels behind the two in registers are streamed: up to 32 panels (most = "auto"; 20 between 6145 and 8191
    columns) it is the library's own choice (fused_variant = 1 asks for the 1024-lane streaming kernel instead), up to 32 it can be
    asked for (fused_variant = 2)."""
    if not 128 < m <= 8192:
        return False
    rows = 64 if m <= 256 else 32 if m <= 512 else 16 if m <= 1024 else 8 if m <= 2048 else 4 if m <= 4096 else 2
    panels = -(-n // rows)
    grid = min(cus, panels, 256)
    if (-(-m // grid) + 3) // 4 * 4 > 64:                    # a workgroup merges a strip of at most 64 columns
        return False
    if m == 2048 or m <= 1024:
        most = 32 if m > 512 else 16 if m > 256 else 8                         # (up to 1024 columns there is no 1024-lane form)
    if most == "auto":
        most = 20 if 6144 < m < 8192 else 32
    return panels <= most * grid


@pytest.mark.parametrize("n,m", SHAPES)
def test_persistent_pass_matches_oracle(fs, oracle, n, m):
    """Both forms of the persistent pass where both apply: the one that streams C every iteration (fused_variant = 1)
    and the one that keeps the workgroup's share of C in LDS and registers (the default where it fits)."""
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    w = W.random_dense(n, m, seed=6000 + n + m, cmax=2.0, eps=0.03)
    iters = 52                                  # one whole block of 50 iterations and a short one
    ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C)
    variants = (0,) if m <= 1024 else (0, 1) if _resident(n, m, cus, most="auto") else (0, 2) if _resident(n, m, cus, most=32) else (0,)
    for variant in variants:
        r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, iters, 0.0, C=dev(w.C), want_f64=True, kernel_mode=6,
                                 fused_variant=variant, time_kernel_every=1)
        assert r["iters"] == iters and not r["nonfinite"]
        assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
        assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
        name = fs.fs_last_kernel_timing()[2]
        assert name == ("k_resident" if (_resident(n, m, cus, most="auto") and variant == 0) or variant == 2 else "k_persist"), \
            (n, m, variant, name)
    assert pot_err(r["f"].cpu().numpy(), ref["f"], w.eps) < TOL_F32
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


def test_persistent_pass_is_the_automatic_choice_and_repeats_bit_for_bit(fs, oracle):
    import torch
    n, m = 700, 3000
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    w = W.random_dense(n, m, seed=6100, cmax=2.0, eps=0.04)
    a, b, C = dev(w.a), dev(w.b), dev(w.C)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert fs.fs_kernel_choice(n, m, 0, True, cus) == "persist"
    r0 = fs.fs_sinkhorn_solve(a, b, w.eps, 60, 0.0, C=C, want_f64=True)
    r6 = fs.fs_sinkhorn_solve(a, b, w.eps, 60, 0.0, C=C, want_f64=True, kernel_mode=6)
    assert torch.equal(r0["f64"], r6["f64"]) and torch.equal(r0["g64"], r6["g64"])
    # no result depends on the order in which workgroups finish or arrive
    for _ in range(3):
        r = fs.fs_sinkhorn_solve(a, b, w.eps, 60, 0.0, C=C, want_f64=True)
        assert torch.equal(r["f64"], r0["f64"]) and torch.equal(r["g"], r0["g"]) and r["marginal_err"] == r0["marginal_err"]
    # the spec entry point takes the same path
    f2, g2, it2 = fs.fs_sinkhorn_dense(C, a, b, w.eps, 60, 0.0)
    assert it2 == 60 and torch.equal(f2, r0["f"]) and torch.equal(g2, r0["g"])
    ref = oracle.solve(w.a, w.b, w.eps, 60, C=w.C)
    assert pot_err(r0["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64


# the streaming form; the resident form (ragged last panel); the resident form with two row groups per workgroup
@pytest.mark.parametrize("n,m", [(320, 1500), (1030, 4096), (1210, 1000), (2500, 500), (5000, 250)])
def test_persistent_pass_stop_rule_history_and_resume(fs, oracle, n, m):
    import torch
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    w = W.random_dense(n, m, seed=6200, eps=0.05)
    a, b, C = dev(w.a), dev(w.b), dev(w.C)
    tol, K = 1e-5, 400
    full = oracle.solve(w.a, w.b, w.eps, K, C=w.C, err_every_iter=True)
    eh = full["err_hist"]
    for c in (1, 7, 10, 40):                     # 40: checks that fall into the second block of a launch sequence
        hist = torch.full((K,), float("nan"), dtype=torch.float32, device="cuda")
        r = fs.fs_sinkhorn_solve(a, b, w.eps, K, tol, C=C, want_f64=True, check_every=c, kernel_mode=6, err_history=hist)
        ks = [k for k in range(c, K + 1, c) if eh[k - 1] < tol]
        assert r["converged"] and r["iters"] == ks[0], (c, r["iters"], ks[0])
        ref = oracle.solve(w.a, w.b, w.eps, r["iters"], C=w.C)
        assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
        assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
        assert abs(r["marginal_err"] - eh[r["iters"] - 1]) <= 1e-3 * eh[r["iters"] - 1] + 5e-7
        h = hist.cpu().numpy()[:r["iters"]]
        assert np.all(np.isfinite(h)) and np.allclose(h, eh[:r["iters"]], rtol=1e-3, atol=5e-7)
    # not reached: runs to max_iter, reports not converged, err of the last iterate
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 15, 1e-30, C=C, check_every=5, kernel_mode=6)
    assert r["iters"] == 15 and not r["converged"]
    assert abs(r["marginal_err"] - eh[14]) <= 1e-3 * eh[14] + 5e-7
    r0 = fs.fs_sinkhorn_solve(a, b, w.eps, 0, 0.0, C=C, kernel_mode=6)
    assert r0["iters"] == 0 and float(r0["f"].abs().max()) == 0.0
    # resume: 13 + 9 iterations against 22 in one go (not bitwise: the hand-over rescales once)
    r1 = fs.fs_sinkhorn_solve(a, b, w.eps, 13, 0.0, C=C, want_f64=True, kernel_mode=6)
    r2 = fs.fs_sinkhorn_solve(a, b, w.eps, 9, 0.0, C=C, want_f64=True, kernel_mode=6, warm_start=True,
                              f64_in=r1["f64"], g64_in=r1["g64"])
    r3 = fs.fs_sinkhorn_solve(a, b, w.eps, 22, 0.0, C=C, want_f64=True, kernel_mode=6)
    assert float((r2["f64"] - r3["f64"]).abs().max()) / w.eps < TOL_F64
    assert float((r2["g64"] - r3["g64"]).abs().max()) / w.eps < TOL_F64
    # in-place warm start through the fp32 potentials
    f, g = r1["f"].clone(), r1["g"].clone()
    r4 = fs.fs_sinkhorn_solve(a, b, w.eps, 9, 0.0, C=C, f=f, g=g, want_f64=True, kernel_mode=6, warm_start=True)
    assert float((r4["f64"] - r3["f64"]).abs().max()) / w.eps < TOL_F32


@pytest.mark.parametrize("eps", [1e-3, 1e-4])
@pytest.mark.parametrize("n,m", [(517, 4100), (300, 4096), (600, 8190), (260, 8192), (300, 12288), (290, 16001), (1500, 3001),
                                 (1100, 1024), (5000, 900), (3000, 512), (6000, 256)])
def test_persistent_pass_small_eps(fs, oracle, n, m, eps):
    """Costs up to 60 at eps 1e-3 and 1e-4: the exact redo of the row phase, and potentials of 10^5 .. 10^6
    in units of eps.  Same bar as the other dense paths in this regime (the iteration does not contract there,
    so the rounding of the 2 K half-steps adds up at worst linearly)."""
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    iters = 300
    w = W.random_dense(n, m, seed=7000 + n + m, cmax=60.0, eps=eps)
    ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C, err_every_iter=True)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, iters, 0.0, C=dev(w.C), want_f64=True, kernel_mode=6)
    assert r["iters"] == iters and not r["nonfinite"]
    df, dg = r["f64"].cpu().numpy() - ref["f"], r["g64"].cpu().numpy() - ref["g"]
    raw = max(np.abs(df).max(), np.abs(dg).max()) / w.eps
    assert raw < TOL_F32, raw
    c = 0.5 * (np.median(df) - np.median(dg))
    e64 = max(np.abs(df - c).max(), np.abs(dg + c).max()) / w.eps
    assert e64 < max(TOL_F64, 2 * iters * 1e-7), (e64, raw)
    assert abs(r["marginal_err"] - ref["err_hist"][-1]) <= 1e-3 * ref["err_hist"][-1] + 5e-7


@pytest.mark.parametrize("eps", [0.05, 2e-3])
@pytest.mark.parametrize("n,m", [(300, 4096), (600, 8192), (290, 16384), (520, 3001), (1300, 1024), (700, 600), (2200, 300), (4400, 200)])
def test_persistent_pass_tiny_and_zero_weights(fs, oracle, n, m, eps):
    """Weights of 1e-30, 1e-36, a denormal and an exact zero in a and b: the columns concerned total less than
    2^-66 in fp32 and go through the exact recomputation inside the merge, every iteration."""
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    w = W.random_dense(n, m, seed=7200 + n + m, cmax=2.0, eps=eps)
    rng = np.random.default_rng(n + m)
    tiny = [1e-30, 1e-36, 1e-41]
    for vec in (w.a, w.b):
        k = vec.shape[0]
        idx = rng.choice(k, size=7, replace=False)
        vec[idx[0]] = 0.0
        for q, j in enumerate(idx[1:]):
            vec[j] = np.float32(tiny[q % 3])
        rest = np.ones(k, dtype=bool)
        rest[idx] = False
        vec[rest] = (vec[rest].astype(np.float64) / vec[rest].sum(dtype=np.float64)).astype(np.float32)
    iters = 40
    ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, iters, 0.0, C=dev(w.C), want_f64=True, kernel_mode=6)
    assert r["iters"] == iters and not r["nonfinite"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-3 * err_ref + 5e-7


@pytest.mark.parametrize("n,m", [(900, 2100), (1030, 4096), (1500, 1024), (3000, 400), (5000, 256)])   # the streaming form; the resident forms
@pytest.mark.parametrize("warm", [False, True])
def test_persistent_pass_gives_up_cleanly_and_the_solve_falls_back(fs, oracle, warm, n, m):
    """wait_limit = 1: a workgroup stops waiting for the others after a single poll, which the host can force
    without any kernel misbehaving (every workgroup still exits).  Asked for by name, the solve then says that
    it gave up (or, with luck, completes); as the library's own choice it is followed by the multi-kernel
    driver and delivers the right answer, also when the start was passed in place."""
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    w = W.random_dense(n, m, seed=6300, cmax=1.0, eps=0.05)
    a, b, C = dev(w.a), dev(w.b), dev(w.C)
    kw, f0, g0 = {}, None, None
    if warm:
        rng = np.random.default_rng(5)
        f0 = (rng.standard_normal(n) * 0.1).astype(np.float32)
        g0 = (rng.standard_normal(m) * 0.1).astype(np.float32)
        kw = dict(f=dev(f0), g=dev(g0), warm_start=True)
    ref = oracle.solve(w.a, w.b, w.eps, 30, C=w.C, f0=f0, g0=g0) if warm else oracle.solve(w.a, w.b, w.eps, 30, C=w.C)
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 30, 0.0, C=C, want_f64=True, wait_limit=1, **kw)
    assert r["iters"] == 30 and not r["nonfinite"] and not r["gave_up"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    outcomes = set()
    for _ in range(4):
        rk = fs.fs_sinkhorn_solve(a, b, w.eps, 30, 0.0, C=C, want_f64=True, kernel_mode=6, wait_limit=1)
        if rk["gave_up"]:
            outcomes.add("gave up")
            assert math.isnan(rk["marginal_err"]) and not rk["converged"]
        else:
            outcomes.add("completed")
            assert rk["iters"] == 30 and not rk["nonfinite"]
    # the next solve on the same workspace is unaffected
    r = fs.fs_sinkhorn_solve(a, b, w.eps, 30, 0.0, C=C, want_f64=True, kernel_mode=6)
    ref = oracle.solve(w.a, w.b, w.eps, 30, C=w.C)
    assert r["iters"] == 30 and not r["nonfinite"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    print("outcomes with wait_limit = 1:", sorted(outcomes))


def test_persistent_pass_rejections(fs):
    import torch
    a = torch.full((100,), 0.01, device="cuda")
    b = torch.full((8192,), 1.0 / 8192, device="cuda")
    C = torch.rand((100, 8192), device="cuda")
    with pytest.raises(fs.FsError, match="kernel_mode 6"):
        fs.fs_sinkhorn_solve(a, b, 0.05, 5, 0.0, C=C, kernel_mode=6)           # 50 panels: strips of 164 columns
    with pytest.raises(fs.FsError, match="kernel_mode 6"):
        fs.fs_sinkhorn_dense_ex(C, a, b, 0.05, 5, 0.0, kernel_mode=6)          # the same through the asynchronous entry
    C16 = torch.rand((300, 4096), device="cuda").to(torch.float16)
    a3 = torch.full((300,), 1.0 / 300, device="cuda")
    b3 = torch.full((4096,), 1.0 / 4096, device="cuda")
    with pytest.raises(fs.FsError, match="kernel_mode 6"):
        fs.fs_sinkhorn_solve(a3, b3, 0.05, 5, 0.0, C=C16, kernel_mode=6)       # fp32 costs only


def _sweep_cases():
    rng = np.random.default_rng(20260511)
    cases = []
    for t in range(34):                          # (from 24 on: the widths with several row groups per workgroup)
        m = int(rng.integers(1025, 16385)) if t < 24 else int(rng.integers(129, 1025))
        n = int(rng.integers(40, 2600)) if t < 24 else int(rng.integers(300, 9000))
        cases.append((t, n, m, float(rng.choice([0.01, 0.03, 0.1])), float(rng.choice([2.0, 20.0])),
                      int(rng.integers(3, 70)), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("t,n,m,eps,cmax,iters,warm", _sweep_cases())
def test_persistent_pass_seeded_shape_sweep(fs, oracle, t, n, m, eps, cmax, iters, warm):
    """Random shapes over the whole range of widths, two cost scales, iteration counts on both sides of a block of
    50, cold and warm starts (the warm start: the oracle's potentials after 5 iterations, given in fp64)."""
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    import torch
    w = W.random_dense(n, m, seed=8100 + t, cmax=cmax, eps=eps)
    kw = {}
    if warm:
        start = oracle.solve(w.a, w.b, w.eps, 5, C=w.C)
        ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C, f0=start["f"], g0=start["g"])
        kw = dict(f=dev(start["f"].astype(np.float32)), g=dev(start["g"].astype(np.float32)), warm_start=True,
                  f64_in=dev(start["f"]), g64_in=dev(start["g"]))
    else:
        ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, iters, 0.0, C=dev(w.C), want_f64=True, kernel_mode=6, **kw)
    assert r["iters"] == iters and not r["nonfinite"]
    tol64 = max(TOL_F64, 2 * iters * 1e-7) if eps * 1e3 < cmax else TOL_F64
    df = r["f64"].cpu().numpy() - ref["f"]
    dg = r["g64"].cpu().numpy() - ref["g"]
    c = 0.5 * (np.median(df) - np.median(dg))
    assert max(np.abs(df).max(), np.abs(dg).max()) / eps < TOL_F32
    assert max(np.abs(df - c).max(), np.abs(dg + c).max()) / eps < tol64, (n, m, eps, cmax, iters, warm)


@pytest.mark.parametrize("n,m,iters", [(65536, 2048, 4), (16384, 8192, 3), (40000, 4096, 3)])
def test_persistent_pass_many_rows(fs, oracle, n, m, iters):
    """Hundreds of panels per workgroup (the shapes the automatic choice takes up to 16384 x 8192 and 65536 x 2048):
    512 MiB of C, every workgroup walks its panels up on even and down on odd iterations."""
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    w = W.random_dense(n, m, seed=8300 + m, cmax=2.0, eps=0.05)
    ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C)
    r = fs.fs_sinkhorn_solve(dev(w.a), dev(w.b), w.eps, iters, 0.0, C=dev(w.C), want_f64=True)
    assert fs.fs_kernel_choice(n, m) == "persist"
    assert r["iters"] == iters and not r["nonfinite"]
    assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
    assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    err_ref = float(oracle.marginal_err(w.a, w.b, w.eps, ref["f"], ref["g"], C=w.C))
    assert abs(r["marginal_err"] - err_ref) <= 1e-4 * err_ref + 5e-7


@pytest.mark.parametrize("n,m,iters", [(600, 8192, 60), (2100, 4096, 52), (300, 3000, 50), (517, 12288, 10)])
def test_persistent_pass_on_request_in_the_asynchronous_solve(fs, oracle, n, m, iters):
    """kernel_mode 6 through fs_sinkhorn_dense_ex (caller workspace, device-side result, no host in the loop): the same
    launches as the blocking solve, so the same bits, and the oracle's potentials; a stop by tolerance ends it too."""
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    import torch
    w = W.random_dense(n, m, seed=8500 + n + m, cmax=2.0, eps=0.04)
    C, a, b = dev(w.C), dev(w.a), dev(w.b)
    ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C)
    r = fs.fs_sinkhorn_solve(a, b, w.eps, iters, 0.0, C=C, kernel_mode=6)
    h = fs.fs_sinkhorn_dense_ex(C, a, b, w.eps, iters, 0.0, kernel_mode=6)
    res = h.result()
    assert res["iters"] == iters and not res["nonfinite"]
    assert torch.equal(h.f, r["f"]) and torch.equal(h.g, r["g"])
    assert pot_err(h.f.cpu().numpy(), ref["f"], w.eps) < TOL_F32
    assert abs(res["marginal_err"] - r["marginal_err"]) == 0.0
    # stop rule on the device: tolerance reached at a check iteration
    tol = float(oracle.solve(w.a, w.b, w.eps, 20, C=w.C, want_err=True, err_every_iter=True)["err_hist"][9]) * 1.5
    tol = max(tol, 2e-6)                        # (the device's error has an fp32 floor of about 1e-7)
    rb = fs.fs_sinkhorn_solve(a, b, w.eps, 200, tol, C=C, kernel_mode=6, check_every=10)
    hb = fs.fs_sinkhorn_dense_ex(C, a, b, w.eps, 200, tol, kernel_mode=6, check_every=10)
    resb = hb.result()
    assert resb["iters"] == rb["iters"] and resb["converged"] and rb["iters"] <= 40
    assert torch.equal(hb.f, rb["f"]) and torch.equal(hb.g, rb["g"])


def test_asynchronous_persistent_solve_reports_an_abandoned_wait(fs, oracle):
    """wait_limit = 1 makes every workgroup stop waiting at once (forced from the host; every workgroup still exits):
    the asynchronous solve has nobody to fall back for it, so it says nonfinite = 2, the launches enqueued behind the
    abandoned one return at once, and the next solve on the same workspace is unaffected."""
    n, m = 600, 8192
    if not _supported(fs, n, m):
        pytest.skip("needs more compute units than this device has")
    import torch
    w = W.random_dense(n, m, seed=8600, cmax=2.0, eps=0.05)
    C, a, b = dev(w.C), dev(w.a), dev(w.b)
    ws = torch.empty(fs.fs_workspace_bytes(n, m, 0), dtype=torch.uint8, device="cuda")
    h = fs.fs_sinkhorn_dense_ex(C, a, b, w.eps, 80, 0.0, workspace=ws, kernel_mode=6, wait_limit=1)
    res = h.result()
    assert res["gave_up"] and res["nonfinite"]
    h2 = fs.fs_sinkhorn_dense_ex(C, a, b, w.eps, 30, 0.0, workspace=ws, kernel_mode=6)
    res2 = h2.result()
    ref = oracle.solve(w.a, w.b, w.eps, 30, C=w.C)
    assert res2["iters"] == 30 and not res2["nonfinite"]
    assert pot_err(h2.f.cpu().numpy(), ref["f"], w.eps) < TOL_F32


@pytest.mark.parametrize("kernel_mode", [6, 2])
def test_ragged_last_panel_with_large_potentials(fs, oracle, kernel_mode):
    """A number of rows that is not a multiple of the panel height, with potentials that are large in units of eps
    (a warm start shifted along the gauge: f - 15, g + 15 at eps = 0.05, so that every V_j exceeds 128 in base-2 units):
    the rows past n of the last panel must contribute exactly nothing.  (They once contributed 2^V_j * 0 = NaN: right
    after the exact repair of every column, but many times slower; hence the comparison of the two solve times beside
    the comparison with the oracle.)"""
    import time
    import torch
    iters = 12
    times = {}
    for n in (1200, 1201):
        if not _supported(fs, n, 4096):
            pytest.skip("needs more compute units than this device has")
        w = W.random_dense(n, 4096, seed=8700, cmax=2.0, eps=0.05)
        C, a, b = dev(w.C), dev(w.a), dev(w.b)
        start = oracle.solve(w.a, w.b, w.eps, 3, C=w.C)
        f0, g0 = start["f"] - 15.0, start["g"] + 15.0
        ref = oracle.solve(w.a, w.b, w.eps, iters, C=w.C, f0=f0, g0=g0)
        kw = dict(warm_start=True, f64_in=dev(f0), g64_in=dev(g0))
        best = 1e9
        for rep in range(4):
            f32, g32 = dev(f0.astype(np.float32)), dev(g0.astype(np.float32))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            r = fs.fs_sinkhorn_solve(a, b, w.eps, iters, 0.0, C=C, f=f32, g=g32, want_f64=True,
                                     kernel_mode=kernel_mode, **kw)
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t0)
        times[n] = best
        assert r["iters"] == iters and not r["nonfinite"]
        assert pot_err(r["f64"].cpu().numpy(), ref["f"], w.eps) < TOL_F64
        assert pot_err(r["g64"].cpu().numpy(), ref["g"], w.eps) < TOL_F64
    assert times[1201] < 2.0 * times[1200] + 2e-4, times
