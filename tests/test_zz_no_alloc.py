"""The entry point that allocates nothing (fs_sinkhorn_dense_static: the solve of fs_sinkhorn_dense_ex on
the library's static scratch buffer) against fs_sinkhorn_dense_ex itself, through the C ABI: the same
kernels run on the same inputs, so the outputs must agree bit for bit.  Two calls in a row on the one
buffer, the second with a smaller problem (the buffer keeps the first call's contents), then a third
that is larger again and takes a different kernel path.
"""
import ctypes

import numpy as np
import pytest

from paper_2605_00837_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fs():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_00837_amd import binding
    return binding


def _both(fs, w, iters, tol, **opt):
    import torch
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    C, a, b = dev(w.C), dev(w.a), dev(w.b)
    # reference: the existing asynchronous entry point with a workspace of the caller's
    h = fs.fs_sinkhorn_dense_ex(C, a, b, w.eps, iters, tol, **opt)
    ref = h.result()
    f_ref, g_ref = h.f.clone(), h.g.clone()
    # the caller passes inputs and outputs only; nothing is allocated inside the call
    f = torch.full((w.n,), float("nan"), dtype=torch.float32, device="cuda")
    g = torch.full((w.m,), float("nan"), dtype=torch.float32, device="cuda")
    res = torch.zeros(16, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    fs.fs_sinkhorn_dense_static(C, a, b, w.eps, iters, tol, f, g, res, **opt)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    got = fs.results_from_device(res.reshape(1, 16))[0]
    assert got["iters"] == ref["iters"] and got["converged"] == ref["converged"] and not got["nonfinite"]
    assert np.float32(got["marginal_err"]).tobytes() == np.float32(ref["marginal_err"]).tobytes()
    assert torch.equal(f, f_ref) and torch.equal(g, g_ref)
    return f.cpu().numpy().astype(np.float64), g.cpu().numpy().astype(np.float64), got


def test_static_scratch_entry_point_matches_the_workspace_one(fs, oracle):
    # 1: fused row-panel kernels + combine, stop rule on the device
    w1 = W.random_dense(1500, 3000, seed=9001, cmax=2.0, eps=0.05)
    f1, g1, r1 = _both(fs, w1, 200, 1e-4, check_every=5)
    assert r1["converged"] and r1["iters"] < 200
    ref = oracle.solve(w1.a, w1.b, w1.eps, r1["iters"], C=w1.C)
    assert max(np.abs(f1 - ref["f"]).max(), np.abs(g1 - ref["g"]).max()) / w1.eps < 1e-3
    # 2: a smaller problem on the same buffer (streaming kernels this time)
    w2 = W.random_dense(130, 517, seed=9002, cmax=2.0, eps=0.05)
    f2, g2, r2 = _both(fs, w2, 40, 0.0, kernel_mode=1)
    ref = oracle.solve(w2.a, w2.b, w2.eps, 40, C=w2.C)
    assert r2["iters"] == 40
    assert max(np.abs(f2 - ref["f"]).max(), np.abs(g2 - ref["g"]).max()) / w2.eps < 1e-3
    # 3: larger again, the one-launch kernel's part of the buffer, 2-byte costs on the way
    w3 = W.random_dense(300, 408, seed=9003, cmax=2.0, eps=0.05)
    _both(fs, w3, 30, 0.0)
    w4 = W.random_dense(64, 8192, seed=9004, cmax=2.0, eps=0.05)
    _both(fs, w4, 12, 0.0)
    # 4: the persistent fused pass on request (its counters and error terms live in the buffer too)
    import torch
    if torch.cuda.get_device_properties(0).multi_processor_count >= 128:
        w5 = W.random_dense(700, 8192, seed=9005, cmax=2.0, eps=0.05)
        f5, g5, r5 = _both(fs, w5, 30, 0.0, kernel_mode=6)
        ref = oracle.solve(w5.a, w5.b, w5.eps, 30, C=w5.C)
        assert max(np.abs(f5 - ref["f"]).max(), np.abs(g5 - ref["g"]).max()) / w5.eps < 1e-3


def test_static_scratch_entry_point_rejects_what_does_not_fit(fs):
    import torch
    n = m = 12288                                    # needs more than the static buffer holds
    assert fs.fs_workspace_bytes(n, m, 0) > fs.FS_STATIC_SCRATCH_BYTES
    z = torch.zeros(16, device="cuda")
    lib = fs._lib
    st = lib.fs_sinkhorn_dense_static(ctypes.c_void_p(z.data_ptr()), ctypes.c_void_p(z.data_ptr()),
                                      ctypes.c_void_p(z.data_ptr()), n, m, 0.05, 10, 0.0, ctypes.c_void_p(z.data_ptr()),
                                      ctypes.c_void_p(z.data_ptr()), None, None, None)
    assert st == fs.FS_ERR_WORKSPACE and "static buffer" in fs.fs_last_error()
