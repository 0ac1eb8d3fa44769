"""Builds libmk.so (HIP kernels + C ABI + host scheduler) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmk.so")
SOURCES = ["mk_api.hip", "mk_kernels.hip", "mk_sched.cpp", "mk_sched.h", "mk_isa.h"]


def lib_path() -> str:
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + [os.path.join(HERE, "..", "include", "mk.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every source for gfx950.  hipcc cross-compiles without a GPU."""
    if not force and not is_stale():
        return LIB
    obj = os.path.join(CSRC, "mk_sched.o")
    host = ["g++", "-O2", "-std=c++17", "-fPIC", "-c", os.path.join(CSRC, "mk_sched.cpp"), "-o", obj]
    dobj = os.path.join(CSRC, "mk_api.o")
    dev = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-c",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-result", "-Wno-inline-asm", os.path.join(CSRC, "mk_api.hip"), "-o", dobj]
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", dobj, obj, "-o", LIB]
    for cmd in (host, dev, link):
        if verbose:
            print(" ".join(cmd))
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
