"""Builds libzz.so (host runtime + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libzz.so")
DEBUG_LIB_PATH = os.path.join(PKG_DIR, "libzz_debug.so")   # the same sources with -DZZ_DEBUG_BOUNDS (checked slot writes)
CLIENT_PATH = os.path.join(PKG_DIR, "zz_c_abi_client")   # the torch-free client of the C ABI (tests/c_abi_client.cpp)
SOURCES = [os.path.join(CSRC, "zz_api.cpp"), os.path.join(CSRC, "zz_transport.cpp"), os.path.join(CSRC, "zz_kernels.hip")]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    """Compile for gfx950.  Packed-FP32 instruction selection is switched off for
    device code (the host pass prints a harmless "not a recognized feature" note).
    Builds the library, its bounds-checking debug variant and the C client."""
    for out, extra in ((LIB_PATH, []), (DEBUG_LIB_PATH, ["-DZZ_DEBUG_BOUNDS"])):
        cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-I" + os.path.join(ROOT, "include"),
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-inline-asm",
               *extra, *SOURCES, "-o", out]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if verbose or res.returncode != 0:
            print(" ".join(cmd))
            print(res.stdout)
            print("\n".join(l for l in res.stderr.splitlines() if "not a recognized feature" not in l))
        if res.returncode != 0:
            raise RuntimeError("hipcc failed building " + os.path.basename(out))
    build_c_client(verbose)
    return LIB_PATH


def build_c_client(verbose: bool = False) -> str:
    """Host-only program that drives libzz.so through include/zz.h with plain hipMalloc memory."""
    cmd = [hipcc(), "-O2", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_client.cpp"), "-L" + PKG_DIR, "-lzz", "-Wl,-rpath,$ORIGIN",
           "-o", CLIENT_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building the C ABI client")
    return CLIENT_PATH


if __name__ == "__main__":
    print(build(verbose=True))
