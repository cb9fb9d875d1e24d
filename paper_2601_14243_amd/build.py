"""Build libjet.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libjet.so")
PROBE_LIB = os.path.join(HERE, "libjet_probe.so")     # measurement aid of bench.py, not part of the product ABI
SOURCES = ["jet_api.hip", "jet_quant.hip", "jet_fused.hip", "jet_gemm.hip"]
PROBE_SOURCES = ["jet_probe.hip"]
HEADERS = ["jet_internal.h", "jet_numerics.h", os.path.join("..", "..", "include", "jet.h")]

# No fast-math: divisions, products and fmas must be the IEEE binary32 operations.
# Packed-fp32 instructions are switched off for the device compiler.
# Only the extern "C" entry points marked JET_API are exported.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(lib: str, sources, force: bool) -> None:
    srcs = [os.path.join(CSRC, s) for s in sources]
    if not force and os.path.exists(lib):
        newest = max(os.path.getmtime(p) for p in srcs + [os.path.join(CSRC, h) for h in HEADERS])
        if os.path.getmtime(lib) >= newest:
            return
    res = subprocess.run(["hipcc", *FLAGS, "-o", lib, *srcs], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)


def build(force: bool = True) -> str:
    """Compile every HIP source: libjet.so (the product) and libjet_probe.so (the benchmark's
    matrix-core rate probe).  Returns the path of libjet.so."""
    _compile(LIB, SOURCES, force)
    _compile(PROBE_LIB, PROBE_SOURCES, force)
    return LIB


if __name__ == "__main__":
    print(build())
