"""Builds libzz.so (host runtime + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libzz.so")
SOURCES = [os.path.join(CSRC, "zz_api.cpp"), os.path.join(CSRC, "zz_transport.cpp"), os.path.join(CSRC, "zz_kernels.hip")]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    """Compile for gfx950.  Packed-FP32 instruction selection is switched off for
    device code (the host pass prints a harmless "not a recognized feature" note)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"),
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-inline-asm",
           *SOURCES, "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "not a recognized feature" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libzz.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
