"""Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblora_gfx950.so")
SOURCES = [os.path.join(CSRC, "lora_host.cpp"), os.path.join(CSRC, "lora_place.cpp"),
           os.path.join(CSRC, "lora_kernels.hip")]
HEADERS = [os.path.join(CSRC, "lora_internal.h"), os.path.join(ROOT, "include", "lora.h"),
           os.path.join(ROOT, "include", "lora_placement.h")]


def build(verbose: bool = False) -> str:
    """Always compiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
           # packed-FP32 instructions stay off in device code (the host pass does not know the flag)
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), "-o", LIB] + SOURCES
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, file=sys.stderr)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))
