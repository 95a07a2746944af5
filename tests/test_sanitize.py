"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the C oracle, and every
host-only path of the library (argument validation of all entry points, workspace arithmetic, the
Section 3.4 selection, the Section 3.3 prompt rule, the Section 3.5 scheduler).  Each is linked into
a small driver under tests/sanitize/ and run as a process of its own: a sanitizer report makes the
driver exit non-zero."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    return r.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-static-libasan", "-Wall", "-Wextra", "-o", exe, os.path.join(HERE, "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "emoe_oracle.c"), "-lm"])
    out = _run([exe], env=dict(ENV, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=0"))   # libgomp's thread pool is not a leak of ours
    assert "oracle driver: ok" in out


def test_host_entry_points_under_sanitizers(tmp_path):
    from paper_2503_06823_amd import build
    hipcc = build._hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.fail("hipcc not found")
    # every -fsanitize= sits directly behind -Xarch_host: the sanitizers instrument the host pass only
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-g", "-O1"]
    objs = build.compile_objects(str(tmp_path / "obj"), extra_flags=san)
    exe = str(tmp_path / "host_driver")
    drv = str(tmp_path / "host_driver.o")
    _run([hipcc, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
          "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"), "-c",
          os.path.join(HERE, "host_driver.cpp"), "-o", drv])
    _run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe, drv,
          *objs])
    out = _run([exe, "300"], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))   # the HIP runtime's own start-up allocations
    assert "rounds ok" in out
