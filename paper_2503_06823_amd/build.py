"""Builds libemoe.so (the HIP kernels and their C ABI) for gfx950 with hipcc.

Objects go to paper_2503_06823_amd/_build/, the library next to this file.  hipcc cross-compiles,
so this runs on a machine without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libemoe.so")

SOURCES = ["api.hip", "maps.hip", "select.hip", "loader.hip", "schedule.hip", "route.hip", "route_mfma.hip", "permute.hip", "combine.hip", "ffn_f32.hip", "ffn_bf16_tiled.hip", "ffn_bf16_mid.hip",
           "ffn_bf16_stream.hip", "peaks.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         # packed fp32 VALU forms are kept out of all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, extra, obj_dir: str = OBJ) -> str:
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 target feature and says so: harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def compile_objects(obj_dir: str, extra_flags=(), jobs: int = 8):
    """Compile every HIP source into `obj_dir` with extra flags (e.g. host-side sanitizers for the
    host-code checks in tests/test_sanitize.py); returns the object paths.  libemoe.so is not touched."""
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        return list(ex.map(lambda s: _compile(s, list(extra_flags), obj_dir), SOURCES))


def build_library(force: bool = True, jobs: int = 8, extra_flags=()) -> str:
    """Compile every HIP source and link libemoe.so; returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, "common.h"), os.path.join(ROOT, "include", "emoe.h")]
    newest_hdr = max(os.path.getmtime(h) for h in headers)

    def need(src):
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        return force or not os.path.exists(obj) or os.path.getmtime(obj) < max(
            os.path.getmtime(os.path.join(CSRC, src)), newest_hdr)

    todo = [s for s in SOURCES if need(s)]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(lambda s: _compile(s, list(extra_flags)), todo))
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    if todo or not os.path.exists(LIB):
        tmp = LIB + f".tmp{os.getpid()}"
        subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(force="--incremental" not in sys.argv))
