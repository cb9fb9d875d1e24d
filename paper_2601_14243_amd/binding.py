"""ctypes binding of libjet.so: argument marshalling only.

``jet_*`` functions mirror include/jet.h one to one (raw pointers, sizes, a
stream handle; they return the status code).  The un-prefixed helpers take
torch CUDA tensors, allocate the outputs with torch, pass ``data_ptr()`` and the
current stream, and raise ``JetError`` on a non-zero status.  No arithmetic of
the method happens in Python, and there is no fallback: if libjet.so is missing
the import of the library fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libjet.so")

JET_SRC_BF16 = 0
JET_SRC_FP8_ROW = 1
GROUP = 128

_lib = None


class JetError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: jet_status {status} ({jet_status_str(status)})")


def lib() -> ctypes.CDLL:
    """Load libjet.so (built in-tree by paper_2601_14243_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2601_14243_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.jet_quant_act.restype = i32
        L.jet_quant_act.argtypes = [vp, vp, i32, i64, i64, vp, vp, vp, vp, vp]
        L.jet_quant_weight.restype = i32
        L.jet_quant_weight.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp]
        for name in ("jet_fp8_linear_fwd", "jet_fp8_linear_dgrad", "jet_fp8_linear_wgrad"):
            f = getattr(L, name)
            f.restype = i32
            f.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp]
        L.jet_rmsnorm_quant.restype = i32
        L.jet_rmsnorm_quant.argtypes = [vp, vp, ctypes.c_float, i64, i64, vp, vp, vp]
        L.jet_silu_mul_quant.restype = i32
        L.jet_silu_mul_quant.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp]
        L.jet_silu_mul_bwd.restype = i32
        L.jet_silu_mul_bwd.argtypes = [vp, vp, i64, vp, i64, i64, vp, vp, i64, vp]
        L.jet_status_str.restype = ctypes.c_char_p
        L.jet_status_str.argtypes = [i32]
        L.jet_version.restype = i32
        _lib = L
    return _lib


# ---------------------------------------------------------------- raw calls

def jet_version() -> int:
    return int(lib().jet_version())


def jet_status_str(status: int) -> str:
    return lib().jet_status_str(int(status)).decode()


def jet_quant_act(x, x_scales, src, M, K, q_row, s_row, q_colT, s_colT, stream) -> int:
    return int(lib().jet_quant_act(x, x_scales, src, M, K, q_row, s_row, q_colT, s_colT, stream))


def jet_quant_weight(w, N, K, q, s, qT, sT, stream) -> int:
    return int(lib().jet_quant_weight(w, N, K, q, s, qT, sT, stream))


def jet_fp8_linear_fwd(qx, sx, qw, sw, y, M, N, K, stream) -> int:
    return int(lib().jet_fp8_linear_fwd(qx, sx, qw, sw, y, M, N, K, stream))


def jet_fp8_linear_dgrad(qdy, sdy, qwT, swT, dx, M, N, K, stream) -> int:
    return int(lib().jet_fp8_linear_dgrad(qdy, sdy, qwT, swT, dx, M, N, K, stream))


def jet_fp8_linear_wgrad(qdyT, sdyT, qxT, sxT, dw, M, N, K, stream) -> int:
    return int(lib().jet_fp8_linear_wgrad(qdyT, sdyT, qxT, sxT, dw, M, N, K, stream))


def jet_rmsnorm_quant(x, gamma, eps, M, K, q_row, s_row, stream) -> int:
    return int(lib().jet_rmsnorm_quant(x, gamma, float(eps), M, K, q_row, s_row, stream))


def jet_silu_mul_quant(gate, up, ld, M, K, q_row, s_row, stream) -> int:
    return int(lib().jet_silu_mul_quant(gate, up, ld, M, K, q_row, s_row, stream))


def jet_silu_mul_bwd(gate, up, ld, dh, M, K, dgate, dup, ld_out, stream) -> int:
    return int(lib().jet_silu_mul_bwd(gate, up, ld, dh, M, K, dgate, dup, ld_out, stream))


# ------------------------------------------------------- tensor conveniences

def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def _need(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or t.dim() != 2:
        raise TypeError(f"{name}: need a contiguous 2-D CUDA tensor of {dtype}")


def quant_act(x: torch.Tensor, x_scales: torch.Tensor | None = None, row: bool = True,
              col: bool = False, out: dict | None = None) -> dict:
    """1x128 quantization of a bf16 [M,K] tensor, or of an FP8-saved one (uint8 codes
    plus x_scales).  Returns dict(q_row, s_row, q_colT, s_colT) with the requested pairs."""
    src = JET_SRC_BF16 if x_scales is None else JET_SRC_FP8_ROW
    _need(x, torch.bfloat16 if src == JET_SRC_BF16 else torch.uint8, "x")
    M, K = x.shape
    dev = x.device
    o = {} if out is None else out
    if row and "q_row" not in o:
        o["q_row"] = torch.empty((M, K), dtype=torch.uint8, device=dev)
        o["s_row"] = torch.empty((M, max(K // GROUP, 1)), dtype=torch.float32, device=dev)
    if col and "q_colT" not in o:
        o["q_colT"] = torch.empty((K, M), dtype=torch.uint8, device=dev)
        o["s_colT"] = torch.empty((K, max(M // GROUP, 1)), dtype=torch.float32, device=dev)
    st = jet_quant_act(_ptr(x), _ptr(x_scales), src, M, K,
                       _ptr(o.get("q_row")) if row else None, _ptr(o.get("s_row")) if row else None,
                       _ptr(o.get("q_colT")) if col else None, _ptr(o.get("s_colT")) if col else None,
                       _stream())
    if st:
        raise JetError(st, "jet_quant_act")
    return o


def _row_pair(M, K, dev, out):
    o = {} if out is None else out
    if "q_row" not in o:
        o["q_row"] = torch.empty((M, K), dtype=torch.uint8, device=dev)
        o["s_row"] = torch.empty((M, max(K // GROUP, 1)), dtype=torch.float32, device=dev)
    return o


def rmsnorm_quant(x: torch.Tensor, gamma: torch.Tensor, eps: float, out: dict | None = None) -> dict:
    """RMSNorm of bf16 [M,K] with bf16 weight [K], written as 1x128 FP8: dict(q_row, s_row)."""
    _need(x, torch.bfloat16, "x")
    M, K = x.shape
    if not gamma.is_cuda or not gamma.is_contiguous() or gamma.dtype != torch.bfloat16 or gamma.shape != (K,):
        raise TypeError("gamma: need a contiguous CUDA bf16 tensor of K elements")
    o = _row_pair(M, K, x.device, out)
    st = jet_rmsnorm_quant(_ptr(x), _ptr(gamma), eps, M, K, _ptr(o["q_row"]), _ptr(o["s_row"]), _stream())
    if st:
        raise JetError(st, "jet_rmsnorm_quant")
    return o


def silu_mul_quant(gate: torch.Tensor, up: torch.Tensor, out: dict | None = None) -> dict:
    """SiLU(gate) * up of two bf16 [M,K] tensors (contiguous, or the two halves of one
    contiguous [M,2K] tensor), written as 1x128 FP8: dict(q_row, s_row)."""
    for t, name in ((gate, "gate"), (up, "up")):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise TypeError(f"{name}: need a 2-D CUDA bf16 tensor with unit column stride")
    if gate.shape != up.shape or gate.stride(0) != up.stride(0):
        raise TypeError("gate and up need one shape and one row stride")
    M, K = gate.shape
    o = _row_pair(M, K, gate.device, out)
    st = jet_silu_mul_quant(_ptr(gate), _ptr(up), gate.stride(0), M, K, _ptr(o["q_row"]), _ptr(o["s_row"]), _stream())
    if st:
        raise JetError(st, "jet_silu_mul_quant")
    return o


def silu_mul_bwd(gate: torch.Tensor, up: torch.Tensor, dh: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """Backward of h = SiLU(gate) * up: returns dgu bf16 [M, 2K] = [dgate | dup] (one contiguous
    tensor, the layout the fused gate/up projection's backward consumes)."""
    for t, name in ((gate, "gate"), (up, "up")):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise TypeError(f"{name}: need a 2-D CUDA bf16 tensor with unit column stride")
    if gate.shape != up.shape or gate.stride(0) != up.stride(0):
        raise TypeError("gate and up need one shape and one row stride")
    _need(dh, torch.bfloat16, "dh")
    M, K = gate.shape
    if tuple(dh.shape) != (M, K):
        raise ValueError("dh: need the shape of gate")
    dgu = torch.empty((M, 2 * K), dtype=torch.bfloat16, device=gate.device) if out is None else out
    _need(dgu, torch.bfloat16, "out")
    if tuple(dgu.shape) != (M, 2 * K):
        raise ValueError("out: need [M, 2K]")
    st = jet_silu_mul_bwd(_ptr(gate), _ptr(up), gate.stride(0), _ptr(dh), M, K, _ptr(dgu),
                          dgu.data_ptr() + 2 * K, 2 * K, _stream())
    if st:
        raise JetError(st, "jet_silu_mul_bwd")
    return dgu


def quant_weight(w: torch.Tensor, transposed: bool = False, out: tuple | None = None):
    """128x128 quantization of bf16 [N,K].  Returns (q, s) or (q, s, qT, sT)."""
    _need(w, torch.bfloat16, "w")
    N, K = w.shape
    dev = w.device
    if out is None:
        q = torch.empty((N, K), dtype=torch.uint8, device=dev)
        s = torch.empty((max(N // GROUP, 1), max(K // GROUP, 1)), dtype=torch.float32, device=dev)
        qT = torch.empty((K, N), dtype=torch.uint8, device=dev) if transposed else None
        sT = torch.empty((max(K // GROUP, 1), max(N // GROUP, 1)), dtype=torch.float32, device=dev) if transposed else None
    else:
        q, s, qT, sT = (tuple(out) + (None, None))[:4]
    st = jet_quant_weight(_ptr(w), N, K, _ptr(q), _ptr(s), _ptr(qT), _ptr(sT), _stream())
    if st:
        raise JetError(st, "jet_quant_weight")
    return (q, s, qT, sT) if transposed else (q, s)


def _need_operand(q, s, rows_per_scale: int, name: str):
    """FP8 codes [rows, R] with their scales [rows / rows_per_scale, R / 128]: the kernels read
    exactly these extents from the raw pointers, so a wrong dtype, a strided view or a scale
    array of another shape is refused here."""
    _need(q, torch.uint8, name)
    _need(s, torch.float32, name + " scales")
    rows, R = q.shape
    if R % GROUP or rows % rows_per_scale:
        raise ValueError(f"{name}: shape {tuple(q.shape)} does not divide into its scale groups")
    if tuple(s.shape) != (rows // rows_per_scale, R // GROUP):
        raise ValueError(f"{name} scales: shape {tuple(s.shape)}, need {(rows // rows_per_scale, R // GROUP)}")
    if s.device != q.device:
        raise ValueError(f"{name}: codes and scales on different devices")


def _gemm_out(out, shape, a, b, name: str) -> torch.Tensor:
    if a.shape[1] != b.shape[1]:
        raise ValueError(f"{name}: reduction lengths differ ({a.shape[1]} and {b.shape[1]})")
    if a.device != b.device:
        raise ValueError(f"{name}: operands on different devices")
    if out is None:
        return torch.empty(shape, dtype=torch.bfloat16, device=a.device)
    _need(out, torch.bfloat16, name + " out")
    if tuple(out.shape) != tuple(shape) or out.device != a.device:
        raise ValueError(f"{name} out: shape {tuple(out.shape)} on {out.device}, need {tuple(shape)} on {a.device}")
    return out


def fp8_linear_fwd(qx, sx, qw, sw, out: torch.Tensor | None = None) -> torch.Tensor:
    """y bf16 [M,N] = X W^T."""
    _need_operand(qx, sx, 1, "qx")
    _need_operand(qw, sw, GROUP, "qw")
    M, K = qx.shape
    N = qw.shape[0]
    y = _gemm_out(out, (M, N), qx, qw, "fp8_linear_fwd")
    st = jet_fp8_linear_fwd(_ptr(qx), _ptr(sx), _ptr(qw), _ptr(sw), _ptr(y), M, N, K, _stream())
    if st:
        raise JetError(st, "jet_fp8_linear_fwd")
    return y


def fp8_linear_dgrad(qdy, sdy, qwT, swT, out: torch.Tensor | None = None) -> torch.Tensor:
    """dx bf16 [M,K] = dY W."""
    _need_operand(qdy, sdy, 1, "qdy")
    _need_operand(qwT, swT, GROUP, "qwT")
    M, N = qdy.shape
    K = qwT.shape[0]
    dx = _gemm_out(out, (M, K), qdy, qwT, "fp8_linear_dgrad")
    st = jet_fp8_linear_dgrad(_ptr(qdy), _ptr(sdy), _ptr(qwT), _ptr(swT), _ptr(dx), M, N, K, _stream())
    if st:
        raise JetError(st, "jet_fp8_linear_dgrad")
    return dx


def fp8_linear_wgrad(qdyT, sdyT, qxT, sxT, out: torch.Tensor | None = None) -> torch.Tensor:
    """dw bf16 [N,K] = dY^T X."""
    _need_operand(qdyT, sdyT, 1, "qdyT")
    _need_operand(qxT, sxT, 1, "qxT")
    N, M = qdyT.shape
    K = qxT.shape[0]
    dw = _gemm_out(out, (N, K), qdyT, qxT, "fp8_linear_wgrad")
    st = jet_fp8_linear_wgrad(_ptr(qdyT), _ptr(sdyT), _ptr(qxT), _ptr(sxT), _ptr(dw), M, N, K, _stream())
    if st:
        raise JetError(st, "jet_fp8_linear_wgrad")
    return dw
