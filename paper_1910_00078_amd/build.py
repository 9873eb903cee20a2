"""Ahead-of-time build of the C-ABI library (libcvx.so) for gfx950 with hipcc.

    python -m paper_1910_00078_amd.build

hipcc cross-compiles without a GPU.  Objects and the shared library are written next to this file
(csrc/_obj/*.o, libcvx.so); they are git-ignored but travel with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_obj")
LIB = os.path.join(HERE, "libcvx.so")
SOURCES = ["cvx_api.cpp", "kernels_direct.hip", "kernels_igemm.hip", "kernels_stem.hip", "kernels_pointwise.hip",
           "kernels_tiled_f32.hip"]
HEADERS = ["cvx_internal.h", "cvx_device.h", os.path.join("..", "..", "include", "cvx.h")]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    "-mllvm", "-amdgpu-mfma-vgpr-form",   # MFMA accumulators stay in VGPRs: no AGPR<->VGPR copies around the k-loop
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _extra_headers():
    return [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".inc"))]


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False, defines=(), lib_path: str = LIB, obj_dir: str = OBJ) -> str:
    """Compile csrc/ into the shared library.  `defines` adds -D flags (developer builds, written to
    another lib_path / obj_dir so the product library is untouched)."""
    return _build(force, verbose, list(defines), lib_path, obj_dir)


def _build(force, verbose, defines, LIB, OBJ) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    hdrs = _extra_headers() + [os.path.join(CSRC, HEADERS[2])]
    jobs = []
    objs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        objs.append(o)
        if force or _stale(o, [s] + hdrs):
            jobs.append([hipcc, "-x", "hip", "-c", s, "-o", o] + FLAGS + ["-D" + d for d in defines])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), r.stdout))
        if verbose and r.stdout.strip():
            print(r.stdout)

    if jobs:
        with ThreadPoolExecutor(max_workers=min(len(jobs), 8)) as ex:
            list(ex.map(run, jobs))
    if jobs or force or _stale(LIB, objs):
        tmp = LIB + ".tmp%d" % os.getpid()
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
