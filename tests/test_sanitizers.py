"""The sanitizer leg, CPU only (never on a GPU machine's device): the oracle and the host side of the library
under AddressSanitizer + UndefinedBehaviorSanitizer.

  * oracle/sanitize_check.c drives every routine of the oracle on small problems that reach its corner cases,
    as one executable with the oracle under -fsanitize=address,undefined;
  * the oracle's pins (tests/test_oracle_pins.py) run once more against a build of the oracle under
    -fsanitize=undefined (a library Python can load without preloading a runtime);
  * tests/host/host_sanitize_check.cpp drives what the C ABI does before it touches a device (validation,
    workspace layout, dispatch table), linked against the library's sources with their HOST code under
    -fsanitize=address,undefined.
Any report makes the program exit non-zero (-fno-sanitize-recover).
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900, **kw)
    assert p.returncode == 0, p.stdout[-4000:]
    return p.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    from oracle import build as ob
    exe, _ = ob.build_sanitized()
    out = _run([exe], env=dict(os.environ, OMP_NUM_THREADS="4"))
    assert "sanitize_check: ok" in out


def test_oracle_pins_against_the_undefined_behaviour_sanitizer_build():
    from oracle import build as ob
    _, lib = ob.build_sanitized()
    env = dict(os.environ, FS_ORACLE_LIB=lib, OMP_NUM_THREADS="4")
    out = _run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                "-p", "no:cacheprovider"], cwd=ROOT, env=env)
    assert " passed" in out and "failed" not in out


def test_host_side_of_the_library_under_sanitizers():
    from paper_2605_00837_amd import build as hb
    exe = hb.build_host_sanitized()
    out = _run([exe])
    assert "host_sanitize_check: ok" in out
