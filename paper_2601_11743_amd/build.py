"""Build libnixie.so for gfx950 in-tree with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libnixie.so")
SOURCES = ["kernels.hip", "runtime.cpp", "hostside.cpp", "planner.cpp", "hostcopy.cpp", "verify.cpp",
           "scheduler.cpp", "spaces.cpp", "vmm.cpp", "placement.cpp"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wextra",
         # packed FP32 instructions are kept out of all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def build(verbose: bool = False) -> str:
    """libnixie.so, then everything that is compiled against its header (the shim and the shim's
    test program), so that the three can never be out of step."""
    lib = build_library(verbose)
    build_shim(verbose)
    return lib


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-shared", "-o", LIB,
           *[os.path.join(CSRC, s) for s in SOURCES], "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed building libnixie.so")
    if verbose and err.strip():
        print(err)
    return LIB


SHIM = os.path.join(HERE, "libnixie_shim.so")
SHIM_APP = os.path.join(ROOT, "tests", "shim_app", "shim_app")


def build_shim(verbose: bool = False) -> str:
    """The LD_PRELOAD shim (host code only; finds libnixie.so beside itself) and the small
    unmodified HIP program the shim's GPU test runs under it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmds = [[hipcc, "-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), "-shared",
             "-o", SHIM, os.path.join(CSRC, "shim.cpp"), "-L" + HERE, "-lnixie", "-Wl,-rpath,$ORIGIN", "-ldl", "-lpthread"],
            [hipcc, "-O2", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-o", SHIM_APP, os.path.join(ROOT, "tests", "shim_app", "shim_app.hip")]]
    for cmd in cmds:
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stderr + "\n")
            raise RuntimeError("hipcc failed: " + cmd[-1])
    return SHIM


if __name__ == "__main__":
    print(build(verbose=True))
