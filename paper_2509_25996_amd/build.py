"""Builds libcast.so (the C-ABI library) in place with hipcc for gfx950.

    python -m paper_2509_25996_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcast.so")
SOURCES = ["cast_api.hip", "adams_step.hip", "select_pack.hip"]
# a stand-alone measurement aid beside the library: bare kernels with the step's streams (csrc/stream_skeleton.hip)
SKELETON = os.path.join(HERE, "stream_skeleton")

# -ffp-contract=off and the correctly rounded divide/sqrt keep every fp32 operation of the
# update a single IEEE-754 rounding; packed fp32 instructions are switched off.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-parameter"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    out = (proc.stdout + proc.stderr)
    # the host pass does not know the device-only target feature and says so: harmless
    out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_library(verbose: bool = False, extra=()) -> str:
    """Compiles the three translation units side by side (objects under _build/, which is not tracked),
    then links libcast.so; the stand-alone stream_skeleton executable is built along."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [["hipcc", *FLAGS, *extra, "-c", "-o", o, os.path.join(CSRC, s)] for s, o in zip(SOURCES, objs)]
    jobs.append(["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                 "-Wall", "-Wextra", "-o", SKELETON, os.path.join(CSRC, "stream_skeleton.hip")])
    with ThreadPoolExecutor(len(jobs)) as pool:
        list(pool.map(lambda cmd: _run(cmd, verbose), jobs))
    _run(["hipcc", "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB, *objs], verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True, extra=sys.argv[1:]))
