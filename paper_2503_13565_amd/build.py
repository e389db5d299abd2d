"""Build the gfx950 shared library ``libmxfp4_hip.so`` in-tree with hipcc.

Run ``python -m paper_2503_13565_amd.build``.  hipcc cross-compiles without a GPU.  Object
files go to ``paper_2503_13565_amd/_build/`` (not committed); the library lands next to this
file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmxfp4_hip.so")
SOURCES = ["api.hip", "cast.hip", "gemv.hip", "gemv_reg.hip", "chain.hip", "mfma.hip", "mfma_tile.hip", "bf16.hip", "e4m3.hip", "e2m3.hip", "mxfmt.hip", "gemm_t.hip", "gemv_tile.hip"]
# packed FP32 instructions are disabled on purpose: see the build notes of this project
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# per file: the leading scalar kernel arguments arrive in scalar registers when a wave starts
PRELOAD = ["-mllvm", "-amdgpu-kernarg-preload-count=16"]
EXTRA = {"gemv_reg.hip": PRELOAD, "gemv_tile.hip": PRELOAD, "chain.hip": PRELOAD, "mfma_tile.hip": PRELOAD, "gemv.hip": PRELOAD, "bf16.hip": PRELOAD}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src: str, verbose: bool, defines=()) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, *EXTRA.get(src, []), *defines, "-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in proc.stderr.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    return obj


def build(verbose: bool = True, jobs: int = 4, knobs: bool = False) -> str:
    """knobs: a measurement build in which the launch-shape switches (environment variables) exist;
    the library as shipped is built without them."""
    os.makedirs(BUILD, exist_ok=True)
    defines = ("-DMXFP4_MEASUREMENT_KNOBS",) if knobs else ()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, verbose, defines), SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(knobs="--knobs" in sys.argv[1:]))
