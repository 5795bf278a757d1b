"""Build libsrft_kv.so (the product) and libsrft_measure.so (measurement aids) in-tree with hipcc, for gfx950.

Every translation unit under csrc/ is compiled to an object of its own (in parallel), then linked; objects whose
source and headers are older than they are are reused unless ``force`` is set.
"""
from __future__ import annotations

import concurrent.futures as cf
import glob
import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libsrft_kv.so")
LIB_MEASURE = os.path.join(PKG, "libsrft_measure.so")
SRC = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "kernels", "*.hip")))
SRC_MEASURE = sorted(glob.glob(os.path.join(CSRC, "measure", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA accumulators in ordinary VGPRs: the vector-ALU tail reads them without v_accvgpr_read copies
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-I", os.path.join(ROOT, "include"),
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd: list[str], verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)


def _object(src: str, force: bool, verbose: bool, extra: list[str]) -> str:
    obj = os.path.join(OBJ, os.path.relpath(src, CSRC).replace(os.sep, "_") + ".o")
    newest = max(os.path.getmtime(f) for f in [src, *HEADERS, os.path.abspath(__file__)])
    if force or not os.path.exists(obj) or os.path.getmtime(obj) < newest:
        _run([hipcc(), *FLAGS, *extra, "-c", src, "-o", obj], verbose)
    return obj


def build(verbose: bool = False, extra: list[str] | None = None, force: bool = True, jobs: int | None = None) -> str:
    """Compile and link both libraries; returns the path of libsrft_kv.so."""
    os.makedirs(OBJ, exist_ok=True)
    extra = list(extra or [])
    jobs = jobs or min(8, os.cpu_count() or 1)
    with cf.ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _object(s, force, verbose, extra), SRC + SRC_MEASURE))
    n = len(SRC)
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs[:n], "-o", LIB], verbose)
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs[n:], "-o", LIB_MEASURE], verbose)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, force="--incremental" not in sys.argv))
