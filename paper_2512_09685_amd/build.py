"""Builds libstar.so (the C-ABI library) in-tree for gfx950.

``python -m paper_2512_09685_amd.build`` or ``build_library()``.  The kernels
are compiled by hipcc with packed-fp32 instructions disabled; the host layer
by g++.  Object files go to ``csrc/_build`` (not committed).
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(PKG, "libstar.so")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument"]
CXX_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__=1",
             "-ffp-contract=off"]
INCLUDES = ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-I" + os.path.join(ROCM, "include")]

HIP_SOURCES = ["star_kernels.hip", "star_reduce_kernels.hip", "star_mfma_kernels.hip", "star_scratch.hip"]
CXX_SOURCES = ["star_api.cpp", "star_plan.cpp", "star_select.cpp"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError("build step failed: " + cmd[-1])
    # hipcc's host pass does not know the packed-fp32 feature and says so; harmless
    noise = [l for l in r.stderr.splitlines() if l.strip() and "packed-fp32-ops" not in l]
    if noise:
        sys.stderr.write("\n".join(noise) + "\n")


def _sources():
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hip", ".cpp"))]
    deps.append(os.path.join(ROOT, "include", "star.h"))
    return deps


def is_current() -> bool:
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in _sources())


def build_library(force: bool = True) -> str:
    if not force and is_current():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.path.join(ROCM, "bin", "hipcc")
    jobs, objs = [], []
    for src in HIP_SOURCES:
        o = os.path.join(OBJ, src + ".o")
        objs.append(o)
        jobs.append([hipcc] + HIP_FLAGS + INCLUDES + ["-c", os.path.join(CSRC, src), "-o", o])
    for src in CXX_SOURCES:
        o = os.path.join(OBJ, src + ".o")
        objs.append(o)
        jobs.append(["g++"] + CXX_FLAGS + INCLUDES + ["-c", os.path.join(CSRC, src), "-o", o])
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(_run, jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs +
         ["-L" + os.path.join(ROCM, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(ROCM, "lib")])
    return LIB


if __name__ == "__main__":
    print(build_library(True))
