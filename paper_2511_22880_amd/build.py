"""Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblora_gfx950.so")
# measurement build: the same library with per-work-group device clocks compiled in (-DLORA_WG_CLOCKS)
LIB_CLOCKS = os.path.join(PKG, "liblora_gfx950_clocks.so")
SOURCES = [os.path.join(CSRC, "lora_host.cpp"), os.path.join(CSRC, "lora_place.cpp"),
           os.path.join(CSRC, "lora_kernels.hip")]
HEADERS = [os.path.join(CSRC, "lora_internal.h"), os.path.join(ROOT, "include", "lora.h"),
           os.path.join(ROOT, "include", "lora_placement.h")]


def build(verbose: bool = False, clocks: bool = False) -> str:
    """Always compiles; returns the path of the shared library.  clocks: the measurement build."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib = LIB_CLOCKS if clocks else LIB
    cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
           # packed-FP32 instructions stay off in device code (the host pass does not know the flag)
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), "-o", lib] + SOURCES
    if clocks:
        cmd.insert(1, "-DLORA_WG_CLOCKS")
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, file=sys.stderr)
    return lib


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True, clocks="--clocks" in sys.argv))
