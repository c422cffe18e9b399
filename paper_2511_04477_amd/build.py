"""Compile libspqt.so (and its benchmark, timeline and test variants) for gfx950 with hipcc, which
cross-compiles without a GPU.

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
# The group-layout GEMV entry points with silent producers and a reducer that waits for a handful of polls only:
# what the tests use to run the give-up path of the exchange (NaN outputs, poison flag) without a stalled kernel.
GIVEUP_LIB = os.path.join(PKG, "libspqt_giveup.so")
GIVEUP_SOURCES = ["pack.cpp", "gemv.hip", "gemv_list.hip", "gemv_bal.hip"]

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


def _jobs(lib: str, sources, defines=(), tag: str = ""):
    """(compile command, ...) per source and the link command of one library."""
    objs = [os.path.join(OBJ, f"{tag}{os.path.splitext(s)[0]}.o") for s in sources]
    common = [_hipcc(), *HIPCC_FLAGS, *[f"-D{d}" for d in defines], "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    compiles = [[*common, "-c", "-o", o, os.path.join(CSRC, s)] for s, o in zip(sources, objs)]
    return compiles, (lib, objs)


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    plan = [_jobs(CALIB_LIB, CALIB_SOURCES),
            _jobs(TIMELINE_LIB, SOURCES, defines=("SPQT_TIMELINE=1",), tag="tl_"),
            _jobs(GIVEUP_LIB, GIVEUP_SOURCES, defines=("SPQT_TEST_GIVE_UP=1",), tag="gu_"),
            _jobs(LIB, SOURCES)]
    # every object of every library in one pool (longest first), then the links
    compiles = sorted((c for cs, _ in plan for c in cs), key=lambda c: -os.path.getsize(c[-1]))
    with ThreadPoolExecutor(JOBS) as pool:
        list(pool.map(lambda c: _run(c, verbose), compiles))
    for _, (lib, objs) in plan:
        tmp = lib + f".tmp{os.getpid()}"
        _run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
        os.replace(tmp, lib)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
