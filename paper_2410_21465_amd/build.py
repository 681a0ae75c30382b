"""Build libshadowkv.so (HIP, gfx950 only) in-tree next to this file.

``python -m paper_2410_21465_amd.build`` compiles unconditionally; ``ensure_built()``
compiles only when the library is missing (used by loaders that must not rebuild).
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libshadowkv.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed fp32 VALU ops are switched off for device code on purpose.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = True) -> str:
    cmd = [HIPCC] + FLAGS + ["-I", os.path.join(_HERE, "..", "include"), "-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if out.strip() and (verbose or res.returncode):
        print(out)
    if res.returncode:
        raise RuntimeError("hipcc failed")
    return LIB


def ensure_built() -> str:
    if not os.path.exists(LIB):
        build_library(verbose=False)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
