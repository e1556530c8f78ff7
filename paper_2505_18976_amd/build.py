"""Builds libgrass.so (all HIP kernels + the C ABI) for gfx950 with hipcc.

The library is built in-tree next to this file; tests, the smoke check and the
benchmark load that file and never build implicitly on a GPU machine.  Every source
is compiled to an object of its own (in parallel, into a temporary directory)
and the objects are linked into one shared library.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libgrass.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers_mtime() -> float:
    deps = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h")) + [__file__]
    return max(os.path.getmtime(d) for d in deps)


def build_library(verbose: bool = True, extra_flags=(), jobs: int | None = None, incremental: bool = False) -> str:
    """incremental=True keeps objects in _build/ and recompiles only sources newer than their object
    (or older than any header); the default compiles everything from scratch."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(8, os.cpu_count() or 1)
    keep = os.path.join(ROOT, "_build")
    if incremental:
        os.makedirs(keep, exist_ok=True)
    with tempfile.TemporaryDirectory(prefix="grass_build_") as scratch:
        tmp = keep if incremental else scratch
        newest_header = _headers_mtime()

        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
                return obj
            cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                   "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE if not verbose else None)
            return obj

        with ThreadPoolExecutor(max_workers=jobs) as pool:
            objects = list(pool.map(compile_one, sources()))
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objects, "-o", LIB_PATH + ".tmp"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    args = sys.argv[1:]
    build_library(incremental="--incremental" in args, extra_flags=[a for a in args if a != "--incremental"])
