"""Build libharp.so (HIP, gfx950) in-tree with hipcc.  ``python -m paper_2605_29843_amd.build``."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libharp.so")

SOURCES = ["harp_api.cpp", "harp_theta.cpp", "harp_kernels.hip", "harp_pipe.hip", "harp_dpp.hip", "harp_mfma.hip",
           "harp_radix.hip", "harp_col.hip", "harp_grad.hip"]
HEADERS = [os.path.join(ROOT, "include", "harp.h"), os.path.join(CSRC, "harp_internal.h")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed-fp32 code generation is switched off for every device function of the library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libharp cannot be built")
    return exe


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS + [os.path.abspath(__file__)]
    return any(os.path.getmtime(p) > t for p in deps)


def build(verbose: bool = True, force: bool = True) -> str:
    """Compile every source of the library for gfx950 and link libharp.so next to this file."""
    if not force and not is_stale():
        return LIB
    objs = []
    bdir = os.path.join(PKG, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for s in SOURCES:
        obj = os.path.join(bdir, os.path.splitext(s)[0] + ".o")
        cmd = [hipcc(), "-x", "hip", "-c", os.path.join(CSRC, s), "-o", obj,
               "-I", os.path.join(ROOT, "include"), "-I", CSRC] + HIPCC_FLAGS
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd)))
        objs.append(obj)
    for s, p in procs:
        if p.wait() != 0:
            raise RuntimeError(f"hipcc failed on {s}")
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(verbose=True, force="--if-stale" not in sys.argv)
    print(LIB)
