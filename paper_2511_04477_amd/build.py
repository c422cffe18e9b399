"""Compile libspqt.so for gfx950 with hipcc (cross-compiles without a GPU).

Every source is compiled to an object of its own, several at a time, and the objects are linked;
objects live in `_build/` next to this file and are rebuilt on every call.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libspqt.so")
SOURCES = ["pack.cpp", "quant_cb.cpp", "gather.hip", "gemv.hip", "gemv_cb.hip", "gemv_cb8.hip", "gemv_cb2.hip", "gemv_list.hip",
           "gemv_bal.hip"]
CALIB_LIB = os.path.join(PKG, "libspqt_calib.so")       # benchmark-only helper kernels
CALIB_SOURCES = ["calib.hip", "baseline_rowmajor.hip"]
# The same kernels with wall-clock stamps per wavefront (python -m paper_2511_04477_amd.timeline).
TIMELINE_LIB = os.path.join(PKG, "libspqt_timeline.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core results stay in ordinary VGPRs: with a separate accumulator file the kernels that use
    # v_mfma would hold their 128 sums twice (AGPRs + copies for the lane folds) and lose a wavefront
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wno-unused-command-line-argument",
]
JOBS = max(1, min(8, os.cpu_count() or 1))


def _hipcc() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return hipcc if os.path.exists(hipcc) else "hipcc"


def _run(cmd, verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(ln for ln in res.stdout.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def _build_one(lib: str, sources, verbose: bool, defines=(), tag: str = "") -> str:
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, f"{tag}{os.path.splitext(s)[0]}.o") for s in sources]
    common = [_hipcc(), *HIPCC_FLAGS, *[f"-D{d}" for d in defines], "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with ThreadPoolExecutor(JOBS) as pool:
        list(pool.map(lambda so: _run([*common, "-c", "-o", so[1], os.path.join(CSRC, so[0])], verbose),
                      zip(sources, objs)))
    tmp = lib + f".tmp{os.getpid()}"
    _run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
    os.replace(tmp, lib)
    return lib


def build(verbose: bool = False) -> str:
    _build_one(CALIB_LIB, CALIB_SOURCES, verbose)
    _build_one(TIMELINE_LIB, SOURCES, verbose, defines=("SPQT_TIMELINE=1",), tag="tl_")
    return _build_one(LIB, SOURCES, verbose)


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
