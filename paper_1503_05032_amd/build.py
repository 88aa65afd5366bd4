"""Builds libcsr5.so (HIP, gfx950) in-tree with hipcc.  No torch involved."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = [os.path.join(PKG, "csrc", "csr5.hip")]
INC = os.path.join(ROOT, "include")
OUT = os.path.join(PKG, "libcsr5.so")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
    "-munsafe-fp-atomics",            # hardware fp64 atomic add (memory is coarse-grained)
    # packed-fp32 instructions are switched off: some forms misbehave on this hardware
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, extra=()) -> str:
    tmp = OUT + f".tmp{os.getpid()}"
    cmd = [hipcc(), *FLAGS, *extra, "-I", INC, "-o", tmp, *SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, OUT)
    return OUT


def is_stale() -> bool:
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    deps = SRC + [os.path.join(INC, "csr5.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    build(extra=sys.argv[1:])
