"""ctypes binding of libjet_probe.so, the benchmark's matrix-core rate probe (a measurement aid
built beside libjet.so; it is not part of the library's ABI and no step of the layer)."""
from __future__ import annotations

import ctypes
import os

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libjet_probe.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is missing: build it with `python -m paper_2601_14243_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.jet_probe_mfma_rate.restype = ctypes.c_int
        L.jet_probe_mfma_rate.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        _lib = L
    return _lib


def jet_probe_mfma_rate(out, workgroups, iters, zero_data, stream) -> int:
    return int(lib().jet_probe_mfma_rate(out, int(workgroups), int(iters), int(zero_data), stream))


def probe_mfma_rate(workgroups: int = 1024, iters: int = 2000, zero_data: bool = False, repeats: int = 5) -> float:
    """Sustained rate (flop/s) of the register-resident FP8 16x16x128 matrix-core stream on the
    current device and stream."""
    out = torch.empty((workgroups * 8,), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    st = jet_probe_mfma_rate(out.data_ptr(), workgroups, max(iters // 10, 1), zero_data, stream)   # warm-up
    if st:
        raise RuntimeError(f"jet_probe_mfma_rate: status {st}")
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(repeats):
        st = jet_probe_mfma_rate(out.data_ptr(), workgroups, iters, zero_data, stream)
        if st:
            raise RuntimeError(f"jet_probe_mfma_rate: status {st}")
    b.record()
    torch.cuda.synchronize()
    flop = float(repeats) * workgroups * 8 * 32 * iters * 65536
    return flop / (a.elapsed_time(b) * 1e-3)
