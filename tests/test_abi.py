"""The C-ABI library builds for gfx950, loads without a GPU, and exports every
symbol that include/fastsinkhorn.h declares (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fastsinkhorn.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2605_00837_amd import build
    if build.is_stale():
        build.build(force=True)
    return ctypes.CDLL(build.LIB)


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fs_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_north_star_entry_points():
    syms = declared_symbols()
    for name in ("fs_sinkhorn_dense", "fs_sinkhorn_points", "fs_plan", "fs_cost"):
        assert name in syms


def test_every_declared_symbol_is_exported(lib):
    syms = declared_symbols()
    assert len(syms) >= 10
    for name in syms:
        assert hasattr(lib, name), f"{name} declared in the header but not exported"


def test_host_only_calls(lib):
    lib.fs_version.restype = ctypes.c_char_p
    lib.fs_last_error.restype = ctypes.c_char_p
    lib.fs_workspace_bytes.restype = ctypes.c_size_t
    lib.fs_workspace_bytes.argtypes = [ctypes.c_int] * 3
    assert lib.fs_version().startswith(b"fastsinkhorn")
    assert lib.fs_last_error() is not None
    dense = lib.fs_workspace_bytes(8192, 8192, 0)
    # potentials + log-weights + column partials: tens of MiB, far below the 256 MiB cost matrix
    assert 1 << 20 < dense < 64 << 20
    assert lib.fs_workspace_bytes(65536, 65536, 3) > 0
    assert lib.fs_workspace_bytes(0, 5, 0) == 0 and lib.fs_workspace_bytes(5, 5, 65) == 0
    assert dense % 256 == 0


def test_binding_mirrors_the_header():
    """Struct layouts and names of the Python binding follow the header (parsed, not imported:
    importing the binding needs torch with a GPU only at call time, so importing is fine here too)."""
    from paper_2605_00837_amd import binding
    assert ctypes.sizeof(binding.fs_result) == 16
    assert ctypes.sizeof(binding.fs_options) == 24 + 5 * 8 + 16
    for name in declared_symbols():
        assert name in binding.EXPORTED and hasattr(binding, name), name


def test_argument_validation_without_gpu(lib):
    """Scalar validation happens before any HIP call, so it can be exercised on a GPU-less host."""
    lib.fs_sinkhorn_dense.restype = ctypes.c_int
    lib.fs_sinkhorn_dense.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int, ctypes.c_int, ctypes.c_float,
                                                              ctypes.c_int, ctypes.c_float] + [ctypes.c_void_p] * 3
    lib.fs_last_error.restype = ctypes.c_char_p
    fake = ctypes.c_void_p(256)
    assert lib.fs_sinkhorn_dense(fake, fake, fake, 0, 4, 0.1, 3, 0.0, fake, fake, None) == -1
    assert b"n and m" in lib.fs_last_error()
    assert lib.fs_sinkhorn_dense(fake, fake, fake, 4, 4, 0.0, 3, 0.0, fake, fake, None) == -1
    assert b"eps" in lib.fs_last_error()
    assert lib.fs_sinkhorn_dense(fake, fake, fake, 4, 4, 0.1, -2, 0.0, fake, fake, None) == -1
    assert lib.fs_sinkhorn_dense(None, fake, fake, 4, 4, 0.1, 3, 0.0, fake, fake, None) == -1
    assert lib.fs_sinkhorn_dense(fake, fake, fake, 4, 4, 0.1, 3, 0.0, None, fake, None) == -1


def test_size_limits_and_new_entry_points_validate_on_the_host(lib):
    """n, m <= FS_MAX_POINTS; batched solves need n, m <= FS_SMALL_MAX and batch >= 1; the barycentric
    mapping takes 1..FS_MAX_BARY_DIM columns: all refused before any HIP call."""
    fake = ctypes.c_void_p(256)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.fs_last_error.restype = ctypes.c_char_p
    lib.fs_sinkhorn_points.restype = ci
    lib.fs_sinkhorn_points.argtypes = [vp, vp, ci, vp, vp, ci, ci, cf, ci, cf, vp, vp, vp]
    assert lib.fs_sinkhorn_points(fake, fake, 3, fake, fake, 1048513, 8, 0.1, 3, 0.0, fake, fake, None) == -1
    assert b"limited" in lib.fs_last_error()
    assert lib.fs_sinkhorn_points(fake, fake, 65, fake, fake, 8, 8, 0.1, 3, 0.0, fake, fake, None) == -1
    lib.fs_sinkhorn_dense_batched.restype = ci
    lib.fs_sinkhorn_dense_batched.argtypes = [vp, vp, vp, ci, ci, ci, cf, ci, cf, vp, vp, vp, vp, vp]
    assert lib.fs_sinkhorn_dense_batched(fake, fake, fake, 0, 8, 8, 0.1, 3, 0.0, fake, fake, None, None, None) == -1
    assert lib.fs_sinkhorn_dense_batched(fake, fake, fake, 2, 257, 8, 0.1, 3, 0.0, fake, fake, None, None, None) == -4
    assert b"256" in lib.fs_last_error()
    lib.fs_barycentric.restype = ci
    lib.fs_barycentric.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, vp, vp, vp, vp, vp, ci, vp, vp]
    assert lib.fs_barycentric(fake, None, None, 0, fake, fake, 4, 4, 0.1, fake, fake, None, None, fake, 5, fake, None) == -1
    assert b"dz" in lib.fs_last_error()
    assert lib.fs_barycentric(fake, None, None, 0, fake, fake, 4, 4, 0.1, fake, None, None, None, fake, 2, fake, None) == -1
    lib.fs_sinkhorn_annealed.restype = ci
    lib.fs_sinkhorn_annealed.argtypes = [vp, vp, vp, ci, vp, vp, ci, ci, cf, cf, cf, ci, ci, cf, vp, vp, vp, vp, vp, vp]
    assert lib.fs_sinkhorn_annealed(fake, None, None, 0, fake, fake, 4, 4, 0.1, 0.05, 0.5, 3, 3, 0.0, fake, fake,
                                    None, None, None, None) == -1
    assert lib.fs_sinkhorn_annealed(fake, None, None, 0, fake, fake, 4, 4, 0.1, 1.0, 1.5, 3, 3, 0.0, fake, fake,
                                    None, None, None, None) == -1


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C (gcc, C11, pedantic) on its own."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "fastsinkhorn.h"\n'
                   "int main(void) { fs_options o; fs_result r; (void)o; (void)r;\n"
                   "  return (int)(sizeof(fs_options) + sizeof(fs_result)) * 0 + FS_DIAG_LEN * 0; }\n")
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run([gcc, "-std=c11", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    # the ctypes mirror of fs_options has the C compiler's layout, field by field
    from paper_2605_00837_amd import binding
    names = [f[0] for f in binding.fs_options._fields_]
    lay = tmp_path / "layout.c"
    lay.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "fastsinkhorn.h"\n'
                   'int main(void) { printf("%zu", sizeof(fs_options));\n' +
                   "".join(f'  printf(" %zu", offsetof(fs_options, {nm}));\n' for nm in names) +
                   "  return 0; }\n")
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c11", "-I", inc, str(lay), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got[0] == ctypes.sizeof(binding.fs_options)
    assert got[1:] == [getattr(binding.fs_options, nm).offset for nm in names]


def test_kernel_choice_table_without_gpu():
    """The dispatch of the solvers is host logic: which kernel takes which shape, pinned here for the five
    benchmark configurations and for the boundaries between the kernels (256 compute units assumed)."""
    from paper_2605_00837_amd import binding as fs
    pick = lambda n, m, d=0, blocking=True, **kw: fs.fs_kernel_choice(n, m, d, blocking, 256, **kw)
    assert pick(256, 256) == "coop"                          # c1
    assert pick(8192, 8192) == "persist"                     # c2
    assert pick(4096, 4096) == "persist"                     # c3: 64 entries per lane do not fit the one-launch kernels
    assert pick(65536, 65536, 3) == "points"                 # c4
    assert pick(16384, 16384, 3) == "points" and pick(16384, 12288) == "fused" and pick(16384, 16384) == "fused"   # c5
    assert pick(64, 64) == "small" and pick(128, 128) == "small" and pick(129, 128) == "coop"
    assert pick(512, 512) == "coop" and pick(513, 512) == "grid" and pick(800, 1024) == "grid"
    assert pick(4096, 128) == "grid" and pick(3000, 256) == "grid" and pick(4096, 2048) == "persist"
    # at more than 128 columns the persistent pass keeps C on the chip and is preferred, unless the problem is small
    assert pick(2048, 2048) == "persist" and pick(2048, 1025) == "persist" and pick(2048, 1024) == "persist"
    assert pick(1024, 1024) == "persist" and pick(4096, 1024) == "persist" and pick(2048, 513) == "persist"
    assert pick(65536, 1024) == "persist" and pick(131072, 600) == "persist" and pick(131073, 600) == "fused"   # 32 panels of 16 rows
    assert pick(4096, 512) == "persist" and pick(4096, 257) == "persist" and pick(131072, 400) == "persist" and pick(131073, 400) == "fused"
    assert pick(4096, 256) == "persist" and pick(131072, 129) == "persist" and pick(131073, 129) != "persist" and pick(65536, 128) != "persist"
    assert pick(256, 2048) == "persist" and pick(800, 1200) == "persist" and pick(640, 1280) == "grid"
    assert pick(300, 1100) == "grid" and pick(200, 2048) == "grid"       # 25 panels: strips of more than 64 columns
    assert pick(2048, 2048, cost_dtype=1) == "grid" and pick(2048, 2048, blocking=False) != "persist"
    assert pick(100, 2048) == "persist"                      # too few rows for that many columns: strips of > 16 columns
    assert pick(40, 20000) == "stream" and pick(30, 16384) == "fused" and pick(30, 16385) == "stream"
    # the persistent fused pass: blocking solves, fp32, 1024 < m <= 8192, strips of at most 64 columns per workgroup
    assert pick(300, 3000) == "persist" and pick(5000, 1100) == "persist" and pick(65536, 2048) == "persist"
    assert pick(8191, 4096) == "persist" and pick(16384, 4096) == "persist"     # panels of 4 rows from 2048 rows up
    assert pick(8192, 8193) == "fused" and pick(8192, 8192, blocking=False) == "fused"
    assert pick(100, 8192) == "fused"                        # 50 panels of 2 rows: strips of 164 columns
    assert pick(254, 8192) == "fused" and pick(255, 8192) == "persist"          # 127 panels: 65 columns; 128 panels: 64
    assert pick(8192, 8192, fused_variant=1) == "fused" and pick(8192, 8192, cost_dtype=1) == "fused"
    assert pick(8192, 8192, kernel_mode=2) == "fused" and pick(8192, 12288, kernel_mode=6) == "persist"
    assert fs.fs_kernel_choice(8192, 8192, 0, True, 64) == "fused"              # 64 compute units: strips of 128 columns
    assert pick(200, 200, 3) == "coop" and pick(1024, 1024, 3) == "grid" and pick(2048, 2048, 3) == "points"
    # asynchronous solves never pick the whole-chip kernel by themselves; a smaller device shrinks its range
    assert pick(1024, 1024, blocking=False) == "fused" and pick(512, 512, blocking=False) == "coop"
    assert pick(1024, 1024, blocking=False, kernel_mode=5) == "grid"
    assert fs.fs_kernel_choice(4096, 128, 0, True, 64) in ("fused", "stream") and fs.fs_kernel_choice(1024, 128, 0, True, 64) == "grid"
    assert fs.fs_kernel_choice(4096, 1024, 0, True, 64) == "persist" and fs.fs_kernel_choice(4096, 1024, 0, True, 8) == "fused"
    # 2-byte costs: fused from 2049 columns on, whole 16-byte chunks only
    assert pick(300, 4096, cost_dtype=1) == "fused" and pick(100, 2048, cost_dtype=1) == "stream"
    assert pick(1000, 1024, cost_dtype=2) == "grid"
    with pytest.raises(fs.FsError, match="m % 8"):
        pick(300, 4100, cost_dtype=1)
    with pytest.raises(fs.FsError, match="kernel_mode 3"):
        pick(300, 300, kernel_mode=3)
    with pytest.raises(fs.FsError, match="kernel_mode 5"):
        pick(4096, 4096, kernel_mode=5)
    with pytest.raises(fs.FsError, match="kernel_mode 6"):
        pick(8192, 8192, blocking=False, kernel_mode=6)
    with pytest.raises(fs.FsError, match="kernel_mode 6"):
        pick(100, 8192, kernel_mode=6)
