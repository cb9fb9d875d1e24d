"""Build libjet.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libjet.so")
SOURCES = ["jet_api.hip", "jet_quant.hip", "jet_fused.hip", "jet_gemm.hip", "jet_probe.hip"]
HEADERS = ["jet_internal.h", "jet_numerics.h", os.path.join("..", "..", "include", "jet.h")]

# No fast-math: divisions, products and fmas must be the IEEE binary32 operations.
# Packed-fp32 instructions are switched off for the device compiler.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(force: bool = True) -> str:
    """Compile every HIP source into libjet.so.  Returns the library path."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in srcs + [os.path.join(CSRC, h) for h in HEADERS])
        if os.path.getmtime(LIB) >= newest:
            return LIB
    cmd = ["hipcc", *FLAGS, "-o", LIB, *srcs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
