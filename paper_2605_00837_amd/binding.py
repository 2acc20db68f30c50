"""Thin ctypes binding of the C-ABI library declared in include/fastsinkhorn.h.

Argument marshalling only: every function takes torch CUDA tensors (PyTorch is
used for device memory and streams, nothing else), hands their ``data_ptr()``
and the current HIP stream to the entry point of the same name, and returns
torch tensors.  There is no CPU fallback: if the shared library is missing the
import of this module fails with instructions to build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastsinkhorn.so")

FS_OK = 0
FS_ERR_INVALID_ARG = -1
FS_ERR_WORKSPACE = -2
FS_ERR_HIP = -3
FS_ERR_UNSUPPORTED = -4


class FsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"fastsinkhorn status {status}: {message}")
        self.status = status


class fs_result(ctypes.Structure):
    _fields_ = [("iters", ctypes.c_int32), ("converged", ctypes.c_int32),
                ("nonfinite", ctypes.c_int32), ("marginal_err", ctypes.c_float)]


class fs_options(ctypes.Structure):
    _fields_ = [("check_every", ctypes.c_int32), ("warm_start", ctypes.c_int32),
                ("kernel_mode", ctypes.c_int32), ("use_graph", ctypes.c_int32),
                ("skip_final_err", ctypes.c_int32), ("fused_variant", ctypes.c_int32),
                ("f64_out", ctypes.c_void_p), ("g64_out", ctypes.c_void_p),
                ("f64_in", ctypes.c_void_p), ("g64_in", ctypes.c_void_p),
                ("err_history", ctypes.c_void_p), ("err_history_len", ctypes.c_int32),
                ("cost_dtype", ctypes.c_int32), ("wait_limit", ctypes.c_int32),
                ("time_kernel_every", ctypes.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built. Run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(or `python paper_2605_00837_amd/build.py`) first; there is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.fs_last_error.restype = ctypes.c_char_p
    lib.fs_version.restype = ctypes.c_char_p
    lib.fs_clear_cache.restype = None
    lib.fs_last_kernel_timing.restype = ci
    lib.fs_last_kernel_timing.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32),
                                          ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_int32)]
    lib.fs_read_rate.restype = ci
    lib.fs_read_rate.argtypes = [vp, ctypes.c_size_t, ci, ctypes.POINTER(ctypes.c_float), vp]
    lib.fs_kernel_choice.restype = ci
    lib.fs_kernel_choice.argtypes = [ci, ci, ci, vp, ci, ci]
    lib.fs_workspace_bytes.restype = ctypes.c_size_t
    lib.fs_workspace_bytes.argtypes = [ci, ci, ci]
    lib.fs_sinkhorn_dense.restype = ci
    lib.fs_sinkhorn_dense.argtypes = [vp, vp, vp, ci, ci, cf, ci, cf, vp, vp, vp]
    lib.fs_sinkhorn_points.restype = ci
    lib.fs_sinkhorn_points.argtypes = [vp, vp, ci, vp, vp, ci, ci, cf, ci, cf, vp, vp, vp]
    lib.fs_sinkhorn_solve.restype = ci
    lib.fs_sinkhorn_solve.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, ci, cf, vp, vp, vp,
                                      ctypes.POINTER(fs_options), ctypes.POINTER(fs_result)]
    lib.fs_sinkhorn_dense_ex.restype = ci
    lib.fs_sinkhorn_dense_ex.argtypes = [vp, vp, vp, ci, ci, cf, ci, cf, vp, vp, vp,
                                         ctypes.POINTER(fs_options), vp, ctypes.c_size_t, vp]
    lib.fs_sinkhorn_dense_static.restype = ci
    lib.fs_sinkhorn_dense_static.argtypes = [vp, vp, vp, ci, ci, cf, ci, cf, vp, vp, vp,
                                             ctypes.POINTER(fs_options), vp]
    lib.fs_sinkhorn_points_ex.restype = ci
    lib.fs_sinkhorn_points_ex.argtypes = [vp, vp, ci, vp, vp, ci, ci, cf, ci, cf, vp, vp, vp,
                                          ctypes.POINTER(fs_options), vp, ctypes.c_size_t, vp]
    for name in ("fs_plan", "fs_cost", "fs_plan_f64", "fs_cost_f64"):
        fn = getattr(lib, name)
        fn.restype = ci
        fn.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, vp, vp, vp, vp]
    lib.fs_sinkhorn_dense_batched.restype = ci
    lib.fs_sinkhorn_dense_batched.argtypes = [vp, vp, vp, ci, ci, ci, cf, ci, cf, vp, vp, vp,
                                              ctypes.POINTER(fs_options), vp]
    lib.fs_sinkhorn_annealed.restype = ci
    lib.fs_sinkhorn_annealed.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, cf, cf, ci, ci, cf, vp, vp, vp,
                                         ctypes.POINTER(fs_options), ctypes.POINTER(fs_result),
                                         ctypes.POINTER(ctypes.c_int32)]
    lib.fs_barycentric.restype = ci
    lib.fs_barycentric.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, vp, vp, vp, vp, vp, ci, vp, vp]
    lib.fs_diagnostics.restype = ci
    lib.fs_diagnostics.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, vp, vp, vp, vp, vp, vp, vp, vp]
    for name in ("fs_update_f", "fs_update_g"):
        fn = getattr(lib, name)
        fn.restype = ci
        fn.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, vp, vp, vp]
    return lib


_lib = _load()

EXPORTED = ("fs_sinkhorn_dense", "fs_sinkhorn_points", "fs_sinkhorn_solve", "fs_workspace_bytes",
            "fs_sinkhorn_dense_ex", "fs_sinkhorn_points_ex", "fs_sinkhorn_dense_static", "fs_sinkhorn_dense_batched", "fs_sinkhorn_annealed", "fs_plan", "fs_cost", "fs_plan_f64",
            "fs_cost_f64", "fs_diagnostics", "fs_barycentric", "fs_update_f", "fs_update_g", "fs_last_error", "fs_clear_cache", "fs_version",
            "fs_last_kernel_timing", "fs_kernel_choice", "fs_read_rate")


def _check(status: int):
    if status < 0:
        raise FsError(status, _lib.fs_last_error().decode())
    return status


def _p(t: Optional[torch.Tensor], dtype=torch.float32):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("expected a CUDA (HIP) tensor")
    if t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    return ctypes.c_void_p(t.data_ptr())


_COST_DTYPES = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}     # FS_COST_F32 / _F16 / _BF16


def _cost(C: Optional[torch.Tensor], opt_kw: dict):
    """Pointer to a dense cost matrix; a 2-byte storage type is recorded in the options (cost_dtype)."""
    if C is None:
        return None
    code = _COST_DTYPES.get(C.dtype)
    if code is None:
        raise TypeError(f"cost matrix must be float32, float16 or bfloat16, got {C.dtype}")
    if code:
        opt_kw["cost_dtype"] = code
    return _p(C, C.dtype)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _shape(C, X, Y, a, b):
    if C is not None:
        n, m = C.shape
        d = 0
    else:
        n, d = X.shape
        m = Y.shape[0]
        if Y.shape[1] != d:
            raise ValueError("X and Y must have the same dimension")
    if a.shape != (n,) or b.shape != (m,):
        raise ValueError("a, b must have shapes (n,), (m,)")
    return int(n), int(m), int(d)


def make_options(check_every=0, warm_start=False, kernel_mode=0, use_graph=0, skip_final_err=False,
                 fused_variant=0, f64_out=None, g64_out=None, f64_in=None, g64_in=None, err_history=None,
                 time_kernel_every=0, cost_dtype=0, wait_limit=0):
    o = fs_options()
    o.cost_dtype = int(cost_dtype)
    o.wait_limit = int(wait_limit)
    o.check_every = int(check_every)
    o.warm_start = int(bool(warm_start))
    o.kernel_mode = int(kernel_mode)
    o.use_graph = int(use_graph)
    o.skip_final_err = int(bool(skip_final_err))
    o.fused_variant = int(fused_variant)
    o.f64_out = _p(f64_out, torch.float64)
    o.g64_out = _p(g64_out, torch.float64)
    o.f64_in = _p(f64_in, torch.float64)
    o.g64_in = _p(g64_in, torch.float64)
    o.err_history = _p(err_history, torch.float32)
    o.err_history_len = 0 if err_history is None else int(err_history.numel())
    o.time_kernel_every = int(time_kernel_every)
    return o


# ---------------------------------------------------------------- entry points, same names as the C ABI
KERNEL_NAMES = {1: "stream", 2: "fused", 3: "small", 4: "coop", 5: "grid", 6: "points", 7: "persist"}


def fs_kernel_choice(n: int, m: int, d: int = 0, blocking: bool = True, compute_units: int = 0, **opt_kw) -> str:
    """Name of the kernel a solve of this shape would run (host logic only; works without a GPU when
    compute_units is given)."""
    o = make_options(**opt_kw)
    return KERNEL_NAMES[_check(_lib.fs_kernel_choice(int(n), int(m), int(d), ctypes.byref(o), int(blocking),
                                                     int(compute_units)))]


def fs_version() -> str:
    return _lib.fs_version().decode()


def fs_last_error() -> str:
    return _lib.fs_last_error().decode()


def fs_clear_cache() -> None:
    _lib.fs_clear_cache()


def fs_last_kernel_timing():
    """(avg_ms per launch, sampled launches, kernel_name, iterations the sampled launches performed) of the
    dominant kernel of the last timed blocking solve."""
    ms, cnt, name, ipl = ctypes.c_float(0), ctypes.c_int32(0), ctypes.c_char_p(), ctypes.c_int32(0)
    _check(_lib.fs_last_kernel_timing(ctypes.byref(ms), ctypes.byref(cnt), ctypes.byref(name), ctypes.byref(ipl)))
    return float(ms.value), int(cnt.value), name.value.decode(), int(ipl.value)


def fs_read_rate(buf, reps: int = 20) -> float:
    """Average microseconds a plain streaming read kernel takes for one pass over the device tensor `buf` (the
    practical read ceiling of the device for a buffer of that size; a measurement aid for benchmarks)."""
    us = ctypes.c_float(0)
    _check(_lib.fs_read_rate(_p(buf, buf.dtype), int(buf.numel() * buf.element_size()), int(reps), ctypes.byref(us), _stream()))
    return float(us.value)


def fs_workspace_bytes(n: int, m: int, d: int = 0) -> int:
    return int(_lib.fs_workspace_bytes(int(n), int(m), int(d)))


def fs_sinkhorn_dense(C, a, b, eps, max_iter, tol, f=None, g=None):
    """Blocking dense solve; returns (f, g, iters)."""
    n, m, _ = _shape(C, None, None, a, b)
    f = torch.empty(n, dtype=torch.float32, device=C.device) if f is None else f
    g = torch.empty(m, dtype=torch.float32, device=C.device) if g is None else g
    it = _check(_lib.fs_sinkhorn_dense(_p(C), _p(a), _p(b), n, m, float(eps), int(max_iter), float(tol),
                                       _p(f), _p(g), _stream()))
    return f, g, it


def fs_sinkhorn_points(X, Y, a, b, eps, max_iter, tol, f=None, g=None):
    """Blocking point-cloud solve; returns (f, g, iters)."""
    n, m, d = _shape(None, X, Y, a, b)
    f = torch.empty(n, dtype=torch.float32, device=X.device) if f is None else f
    g = torch.empty(m, dtype=torch.float32, device=X.device) if g is None else g
    it = _check(_lib.fs_sinkhorn_points(_p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), int(max_iter),
                                        float(tol), _p(f), _p(g), _stream()))
    return f, g, it


def fs_sinkhorn_solve(a, b, eps, max_iter, tol, C=None, X=None, Y=None, f=None, g=None, want_f64=False,
                      **opt_kw):
    """Blocking solve with options.  Returns dict(f, g, iters, converged, nonfinite, marginal_err[, f64, g64])."""
    n, m, d = _shape(C, X, Y, a, b)
    dev = a.device
    f = torch.empty(n, dtype=torch.float32, device=dev) if f is None else f
    g = torch.empty(m, dtype=torch.float32, device=dev) if g is None else g
    f64 = g64 = None
    if want_f64:
        f64 = torch.empty(n, dtype=torch.float64, device=dev)
        g64 = torch.empty(m, dtype=torch.float64, device=dev)
        opt_kw.update(f64_out=f64, g64_out=g64)
    Cp = _cost(C, opt_kw)
    o = make_options(**opt_kw)
    res = fs_result()
    it = _check(_lib.fs_sinkhorn_solve(Cp, _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), int(max_iter),
                                       float(tol), _p(f), _p(g), _stream(), ctypes.byref(o), ctypes.byref(res)))
    out = dict(f=f, g=g, iters=it, converged=bool(res.converged), nonfinite=bool(res.nonfinite),
               gave_up=res.nonfinite == 2, marginal_err=float(res.marginal_err))
    if want_f64:
        out.update(f64=f64, g64=g64)
    return out


def fs_sinkhorn_annealed(a, b, eps, eps_start, decay, stage_iters, max_iter, tol, C=None, X=None, Y=None,
                         f=None, g=None, want_f64=False, **opt_kw):
    """eps-scaling: stages at eps_start * decay^k > eps (stage_iters iterations each, warm-started), then
    the final stage at eps.  Returns the dict of fs_sinkhorn_solve plus total_iters."""
    n, m, d = _shape(C, X, Y, a, b)
    dev = a.device
    f = torch.zeros(n, dtype=torch.float32, device=dev) if f is None else f
    g = torch.zeros(m, dtype=torch.float32, device=dev) if g is None else g
    f64 = g64 = None
    if want_f64:
        f64 = torch.empty(n, dtype=torch.float64, device=dev)
        g64 = torch.empty(m, dtype=torch.float64, device=dev)
        opt_kw.update(f64_out=f64, g64_out=g64)
    Cp = _cost(C, opt_kw)
    o = make_options(**opt_kw)
    res = fs_result()
    total = ctypes.c_int32(0)
    it = _check(_lib.fs_sinkhorn_annealed(Cp, _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), float(eps_start),
                                          float(decay), int(stage_iters), int(max_iter), float(tol), _p(f), _p(g),
                                          _stream(), ctypes.byref(o), ctypes.byref(res), ctypes.byref(total)))
    out = dict(f=f, g=g, iters=it, total_iters=int(total.value), converged=bool(res.converged),
               nonfinite=bool(res.nonfinite), marginal_err=float(res.marginal_err))
    if want_f64:
        out.update(f64=f64, g64=g64)
    return out


def _result_from_device(t: torch.Tensor):
    raw = t.cpu().numpy().tobytes()
    r = fs_result.from_buffer_copy(raw)
    return dict(iters=int(r.iters), converged=bool(r.converged), nonfinite=bool(r.nonfinite),
                gave_up=r.nonfinite == 2, marginal_err=float(r.marginal_err))


class AsyncSolve:
    """Handle of an asynchronous (_ex) solve: tensors stay alive until read."""

    def __init__(self, f, g, result_dev, workspace, keep):
        self.f, self.g, self.result_dev, self.workspace, self._keep = f, g, result_dev, workspace, keep

    def result(self):
        """Synchronises with the device and returns the fs_result as a dict."""
        return _result_from_device(self.result_dev)


def _ex(fn_dense: bool, C, X, Y, a, b, eps, max_iter, tol, f, g, workspace, opt_kw):
    n, m, d = _shape(C, X, Y, a, b)
    dev = a.device
    f = torch.empty(n, dtype=torch.float32, device=dev) if f is None else f
    g = torch.empty(m, dtype=torch.float32, device=dev) if g is None else g
    need = fs_workspace_bytes(n, m, d)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    res = torch.zeros(16, dtype=torch.uint8, device=dev)
    Cp = _cost(C, opt_kw)
    o = make_options(**opt_kw)
    if fn_dense:
        st = _lib.fs_sinkhorn_dense_ex(Cp, _p(a), _p(b), n, m, float(eps), int(max_iter), float(tol), _p(f),
                                       _p(g), _stream(), ctypes.byref(o), _p(workspace, torch.uint8),
                                       workspace.numel(), _p(res, torch.uint8))
    else:
        st = _lib.fs_sinkhorn_points_ex(_p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), int(max_iter),
                                        float(tol), _p(f), _p(g), _stream(), ctypes.byref(o),
                                        _p(workspace, torch.uint8), workspace.numel(), _p(res, torch.uint8))
    _check(st)
    return AsyncSolve(f, g, res, workspace, (C, X, Y, a, b, opt_kw))


def fs_sinkhorn_dense_ex(C, a, b, eps, max_iter, tol, f=None, g=None, workspace=None, **opt_kw) -> AsyncSolve:
    """Asynchronous dense solve on the current stream (no host synchronisation)."""
    return _ex(True, C, None, None, a, b, eps, max_iter, tol, f, g, workspace, opt_kw)


FS_STATIC_SCRATCH_BYTES = 20 << 20


def fs_sinkhorn_dense_static(C, a, b, eps, max_iter, tol, f, g, result_dev, **opt_kw) -> None:
    """Asynchronous dense solve on the library's static scratch buffer; the C call allocates nothing.  The
    caller supplies every output: f [n], g [m] fp32 and result_dev, a uint8 tensor of 16 bytes (decode with
    results_from_device after synchronising)."""
    n, m, _ = _shape(C, None, None, a, b)
    Cp = _cost(C, opt_kw)
    o = make_options(**opt_kw)
    _check(_lib.fs_sinkhorn_dense_static(Cp, _p(a), _p(b), n, m, float(eps), int(max_iter), float(tol), _p(f),
                                         _p(g), _stream(), ctypes.byref(o), _p(result_dev, torch.uint8)))


def fs_sinkhorn_points_ex(X, Y, a, b, eps, max_iter, tol, f=None, g=None, workspace=None, **opt_kw) -> AsyncSolve:
    """Asynchronous point-cloud solve on the current stream (no host synchronisation)."""
    return _ex(False, None, X, Y, a, b, eps, max_iter, tol, f, g, workspace, opt_kw)


def fs_sinkhorn_dense_batched(C, a, b, eps, max_iter, tol, f=None, g=None, want_f64=False, **opt_kw):
    """`batch` small dense problems of one shape in one launch (C [B, n, m], a [B, n], b [B, m]; n, m <= 256).
    Asynchronous.  Returns dict(f [B, n], g [B, m], result = uint8 tensor [B, 16] of fs_result records
    (decode with results_from_device)[, f64, g64])."""
    if C.dim() != 3 or a.dim() != 2 or b.dim() != 2:
        raise ValueError("expected C [B, n, m], a [B, n], b [B, m]")
    B, n, m = (int(x) for x in C.shape)
    if tuple(a.shape) != (B, n) or tuple(b.shape) != (B, m):
        raise ValueError("a, b must have shapes (B, n), (B, m)")
    dev = C.device
    f = torch.empty((B, n), dtype=torch.float32, device=dev) if f is None else f
    g = torch.empty((B, m), dtype=torch.float32, device=dev) if g is None else g
    out = dict(f=f, g=g)
    if want_f64:
        out["f64"] = torch.empty((B, n), dtype=torch.float64, device=dev)
        out["g64"] = torch.empty((B, m), dtype=torch.float64, device=dev)
        opt_kw.update(f64_out=out["f64"], g64_out=out["g64"])
    Cp = _cost(C, opt_kw)
    o = make_options(**opt_kw)
    res = torch.zeros((B, 16), dtype=torch.uint8, device=dev)
    _check(_lib.fs_sinkhorn_dense_batched(Cp, _p(a), _p(b), B, n, m, float(eps), int(max_iter), float(tol),
                                          _p(f), _p(g), _stream(), ctypes.byref(o), _p(res, torch.uint8)))
    out["result"] = res
    return out


def results_from_device(t: torch.Tensor):
    """Decode a [B, 16] uint8 tensor of fs_result records (synchronises)."""
    raw = t.cpu().numpy()
    return [_result_from_device(torch.from_numpy(raw[q].copy())) for q in range(raw.shape[0])]


def _pots(f, g):
    if f.dtype == torch.float64:
        return torch.float64
    return torch.float32


def fs_plan(a, b, eps, f, g, C=None, X=None, Y=None, P=None):
    """P[i, j] = a_i b_j exp((f_i + g_j - C_ij)/eps) as an fp32 n x m tensor (fp32 or fp64 potentials)."""
    n, m, d = _shape(C, X, Y, a, b)
    P = torch.empty((n, m), dtype=torch.float32, device=a.device) if P is None else P
    dt = _pots(f, g)
    fn = _lib.fs_plan_f64 if dt == torch.float64 else _lib.fs_plan
    _check(fn(_p(C), _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), _p(f, dt), _p(g, dt), _p(P), _stream()))
    return P


def fs_cost(a, b, eps, f, g, C=None, X=None, Y=None):
    """<C, P> as a 1-element fp64 device tensor (fp32 or fp64 potentials)."""
    n, m, d = _shape(C, X, Y, a, b)
    out = torch.empty(1, dtype=torch.float64, device=a.device)
    dt = _pots(f, g)
    fn = _lib.fs_cost_f64 if dt == torch.float64 else _lib.fs_cost
    _check(fn(_p(C), _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), _p(f, dt), _p(g, dt),
              _p(out, torch.float64), _stream()))
    return out


fs_plan_f64 = fs_plan
fs_cost_f64 = fs_cost

def fs_barycentric(a, b, eps, f, g, Z, C=None, X=None, Y=None):
    """T[i] = sum_j P_ij Z[j] / sum_j P_ij for the plan of (f, g); Z is [m, dz] fp32, dz <= 4.  Returns [n, dz]."""
    n, m, d = _shape(C, X, Y, a, b)
    if Z.dim() != 2 or Z.shape[0] != m:
        raise ValueError("Z must be [m, dz]")
    dz = int(Z.shape[1])
    dt = _pots(f, g)
    T = torch.empty((n, dz), dtype=torch.float32, device=a.device)
    f32 = (_p(f), _p(g)) if dt == torch.float32 else (None, None)
    f64 = (_p(f, dt), _p(g, dt)) if dt == torch.float64 else (None, None)
    _check(_lib.fs_barycentric(_p(C), _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), f32[0], f32[1], f64[0], f64[1],
                               _p(Z), dz, _p(T), _stream()))
    return T


DIAG_FIELDS = ("cost", "mass", "kl", "primal", "dual", "row_err", "col_err")


def fs_diagnostics(a, b, eps, f, g, C=None, X=None, Y=None, want_marginals=False):
    """Cost, mass, KL, primal and dual objectives and both marginal L1 errors of the plan of (f, g), in
    one pass.  Returns dict(out=fp64 device tensor of 8 values in the order of DIAG_FIELDS (FS_DIAG_* in
    the header), row_marginal, col_marginal = fp64 device tensors, or None when not asked for)."""
    n, m, d = _shape(C, X, Y, a, b)
    dt = _pots(f, g)
    out = torch.empty(8, dtype=torch.float64, device=a.device)
    r = torch.empty(n, dtype=torch.float64, device=a.device) if want_marginals else None
    c = torch.empty(m, dtype=torch.float64, device=a.device) if want_marginals else None
    f32 = (_p(f), _p(g)) if dt == torch.float32 else (None, None)
    f64 = (_p(f, dt), _p(g, dt)) if dt == torch.float64 else (None, None)
    _check(_lib.fs_diagnostics(_p(C), _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), f32[0], f32[1], f64[0], f64[1],
                               _p(out, torch.float64), _p(r, torch.float64), _p(c, torch.float64), _stream()))
    return dict(out=out, row_marginal=r, col_marginal=c)


def fs_update_f(a, b, eps, g64, C=None, X=None, Y=None):
    """One f half-step (Eq. 9) from fp64 g; returns fp64 f."""
    n, m, d = _shape(C, X, Y, a, b)
    out = torch.empty(n, dtype=torch.float64, device=a.device)
    _check(_lib.fs_update_f(_p(C), _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), _p(g64, torch.float64),
                            _p(out, torch.float64), _stream()))
    return out


def fs_update_g(a, b, eps, f64, C=None, X=None, Y=None):
    """One g half-step (Eq. 10) from fp64 f; returns fp64 g."""
    n, m, d = _shape(C, X, Y, a, b)
    out = torch.empty(m, dtype=torch.float64, device=a.device)
    _check(_lib.fs_update_g(_p(C), _p(X), _p(Y), d, _p(a), _p(b), n, m, float(eps), _p(f64, torch.float64),
                            _p(out, torch.float64), _stream()))
    return out
