"""CPU oracle of the block-scaled FP8 linear layer (test infrastructure only).

A ctypes view of ``liboracle.so`` (built from ``jet_oracle.c`` with gcc).  Only
tests, the smoke check and the benchmark's CPU-baseline leg import this package;
the GPU library never does, and this package never imports the GPU library.

All arrays are host numpy arrays.  bf16 tensors are ``uint16`` arrays holding
the bf16 bit patterns; FP8 tensors are ``uint8`` arrays of E4M3 codes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jet_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

SRC_BF16 = 0
SRC_FP8_ROW = 1
SB_BLOCK = 0
SB_ROW = 1
GROUP = 128

ERRORS = {1: "null", 2: "shape", 4: "arg", 6: "non-finite input"}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.orc_num_threads.restype = i32
        L.orc_set_num_threads.argtypes = [i32]
        L.orc_e4m3_decode.restype = ctypes.c_float
        L.orc_e4m3_decode.argtypes = [ctypes.c_uint8]
        L.orc_e4m3_encode.restype = ctypes.c_uint8
        L.orc_e4m3_encode.argtypes = [ctypes.c_float]
        L.orc_bf16_rne.restype = ctypes.c_uint16
        L.orc_bf16_rne.argtypes = [ctypes.c_float]
        L.orc_e4m3_encode_n.argtypes = [vp, vp, i64]
        L.orc_e4m3_decode_n.argtypes = [vp, vp, i64]
        L.orc_bf16_rne_n.argtypes = [vp, vp, i64]
        L.orc_quant_act.restype = i32
        L.orc_quant_act.argtypes = [vp, vp, i32, i64, i64, vp, vp, vp, vp]
        L.orc_quant_weight.restype = i32
        L.orc_quant_weight.argtypes = [vp, i64, i64, vp, vp, vp, vp]
        L.orc_gemm.restype = i32
        L.orc_gemm.argtypes = [vp, vp, vp, vp, i32, i64, i64, i64, vp, i64, vp, i64, vp, vp, vp, vp, vp]
        for name in ("orc_fp8_linear_fwd", "orc_fp8_linear_dgrad", "orc_fp8_linear_wgrad"):
            f = getattr(L, name)
            f.restype = i32
            f.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp]
        L.orc_bf16_from_double.restype = ctypes.c_uint16
        L.orc_bf16_from_double.argtypes = [ctypes.c_double]
        L.orc_silu_bf16.restype = ctypes.c_uint16
        L.orc_silu_bf16.argtypes = [ctypes.c_uint16]
        L.orc_rmsnorm.restype = i32
        L.orc_rmsnorm.argtypes = [vp, vp, ctypes.c_float, i64, i64, vp]
        L.orc_silu_mul.restype = i32
        L.orc_silu_mul.argtypes = [vp, vp, i64, i64, i64, vp]
        L.orc_silu_grad.restype = ctypes.c_double
        L.orc_silu_grad.argtypes = [ctypes.c_double]
        L.orc_silu_mul_bwd.restype = i32
        L.orc_silu_mul_bwd.argtypes = [vp, vp, i64, vp, i64, i64, vp, vp, i64]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(int(n))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc: int):
    if rc != 0:
        raise ValueError(f"oracle error {rc}: {ERRORS.get(rc, '?')}")


# ------------------------------------------------------------------ formats

def e4m3_decode(codes) -> np.ndarray:
    c = _c(codes, np.uint8)
    out = np.empty(c.shape, np.float32)
    lib().orc_e4m3_decode_n(_p(c), _p(out), c.size)
    return out


def e4m3_encode(t) -> np.ndarray:
    t = _c(t, np.float32)
    out = np.empty(t.shape, np.uint8)
    lib().orc_e4m3_encode_n(_p(t), _p(out), t.size)
    return out


def bf16_rne(v) -> np.ndarray:
    v = _c(v, np.float32)
    out = np.empty(v.shape, np.uint16)
    lib().orc_bf16_rne_n(_p(v), _p(out), v.size)
    return out


def bf16_to_f32(h) -> np.ndarray:
    h = _c(h, np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------- quantizers

def quant_act(x, x_scales=None, src=SRC_BF16, row=True, col=False):
    """1x128 quantization.  Returns dict with q_row,s_row and/or q_colT,s_colT."""
    x = _c(x, np.uint16 if src == SRC_BF16 else np.uint8)
    M, K = x.shape
    xs = None if x_scales is None else _c(x_scales, np.float32)
    out = {}
    q_row = s_row = q_colT = s_colT = None
    if row:
        q_row = np.empty((M, K), np.uint8)
        s_row = np.empty((M, max(K // GROUP, 1)), np.float32)
    if col:
        q_colT = np.empty((K, M), np.uint8)
        s_colT = np.empty((K, max(M // GROUP, 1)), np.float32)
    _check(lib().orc_quant_act(_p(x), _p(xs), src, M, K, _p(q_row), _p(s_row), _p(q_colT),
                               _p(s_colT)))
    if row:
        out["q_row"], out["s_row"] = q_row, s_row
    if col:
        out["q_colT"], out["s_colT"] = q_colT, s_colT
    return out


def quant_weight(w, transposed=False):
    """128x128 quantization.  Returns (q, s) or (q, s, qT, sT)."""
    w = _c(w, np.uint16)
    N, K = w.shape
    q = np.empty((N, K), np.uint8)
    s = np.empty((max(N // GROUP, 1), max(K // GROUP, 1)), np.float32)
    qT = sT = None
    if transposed:
        qT = np.empty((K, N), np.uint8)
        sT = np.empty((max(K // GROUP, 1), max(N // GROUP, 1)), np.float32)
    _check(lib().orc_quant_weight(_p(w), N, K, _p(q), _p(s), _p(qT), _p(sT)))
    return (q, s, qT, sT) if transposed else (q, s)


# --------------------------------------------------------------------- GEMM

def gemm(a, sa, b, sb, sb_mode=SB_BLOCK, rows=None, cols=None, want_exact=True):
    """OUT[i,j] = sum_r A[i,r] B[j,r] on block-scaled FP8 operands.

    Returns dict(acc=f32 reference-order result, out=bf16 bits, exact=f64
    order-independent value, sum_abs=f64 sum of |group terms|, sum_abs_prod=f64
    sum of |single products| times the group scales), compact over the requested
    rows / cols."""
    a, b = _c(a, np.uint8), _c(b, np.uint8)
    sa, sb = _c(sa, np.float32), _c(sb, np.float32)
    I, R = a.shape
    J, R2 = b.shape
    if R != R2:
        raise ValueError("reduction lengths differ")
    r = None if rows is None else _c(rows, np.int64)
    c = None if cols is None else _c(cols, np.int64)
    nr = I if r is None else r.size
    nc = J if c is None else c.size
    acc = np.empty((nr, nc), np.float32)
    out = np.empty((nr, nc), np.uint16)
    exact = np.empty((nr, nc), np.float64) if want_exact else None
    sabs = np.empty((nr, nc), np.float64) if want_exact else None
    sprod = np.empty((nr, nc), np.float64) if want_exact else None
    _check(lib().orc_gemm(_p(a), _p(sa), _p(b), _p(sb), sb_mode, I, J, R, _p(r), nr, _p(c), nc,
                          _p(acc), _p(out), _p(exact), _p(sabs), _p(sprod)))
    return {"acc": acc, "out": out, "exact": exact, "sum_abs": sabs, "sum_abs_prod": sprod}


def _named(fn, a, sa, b, sb, M, N, K, oshape):
    a, b = _c(a, np.uint8), _c(b, np.uint8)
    sa, sb = _c(sa, np.float32), _c(sb, np.float32)
    acc = np.empty(oshape, np.float32)
    out = np.empty(oshape, np.uint16)
    _check(fn(_p(a), _p(sa), _p(b), _p(sb), M, N, K, _p(acc), _p(out)))
    return acc, out


def fp8_linear_fwd(qx, sx, qw, sw):
    """Y[M,N] = X W^T.  Returns (acc f32, y bf16 bits)."""
    M, K = np.shape(qx)
    N = np.shape(qw)[0]
    return _named(lib().orc_fp8_linear_fwd, qx, sx, qw, sw, M, N, K, (M, N))


def fp8_linear_dgrad(qdy, sdy, qwT, swT):
    """dX[M,K] = dY W.  Returns (acc f32, dx bf16 bits)."""
    M, N = np.shape(qdy)
    K = np.shape(qwT)[0]
    return _named(lib().orc_fp8_linear_dgrad, qdy, sdy, qwT, swT, M, N, K, (M, K))


def fp8_linear_wgrad(qdyT, sdyT, qxT, sxT):
    """dW[N,K] = dY^T X.  Returns (acc f32, dw bf16 bits)."""
    N, M = np.shape(qdyT)
    K = np.shape(qxT)[0]
    return _named(lib().orc_fp8_linear_wgrad, qdyT, sdyT, qxT, sxT, M, N, K, (N, K))


# ---------------------------------------------------------- fused producers

def bf16_from_double(v: float) -> int:
    return int(lib().orc_bf16_from_double(float(v)))


def silu_bf16(g_bits: int) -> int:
    """bf16( silu(g) ) for one bf16 bit pattern."""
    return int(lib().orc_silu_bf16(int(g_bits)))


def rmsnorm(x, gamma, eps):
    """h = bf16(gamma * bf16(x * rsqrt(mean(x^2) + eps))) as bf16 bits [M,K]."""
    x, gamma = _c(x, np.uint16), _c(gamma, np.uint16)
    M, K = x.shape
    if gamma.shape != (K,):
        raise ValueError("gamma must have K elements")
    h = np.empty((M, K), np.uint16)
    _check(lib().orc_rmsnorm(_p(x), _p(gamma), float(eps), M, K, _p(h)))
    return h


def silu_mul(gate, up):
    """h = bf16(bf16(silu(gate)) * up) as bf16 bits [M,K]; gate and up may be views of one
    [M, 2K] array (equal row strides)."""
    gate, up = np.asarray(gate), np.asarray(up)
    if gate.dtype != np.uint16 or up.dtype != np.uint16 or gate.shape != up.shape:
        raise ValueError("gate and up must be uint16 arrays of one shape")
    M, K = gate.shape
    if gate.strides != up.strides or gate.strides[1] != 2 or gate.strides[0] % 2:
        raise ValueError("gate and up need unit column stride and a common row stride")
    ld = gate.strides[0] // 2
    h = np.empty((M, K), np.uint16)
    _check(lib().orc_silu_mul(gate.ctypes.data_as(ctypes.c_void_p), up.ctypes.data_as(ctypes.c_void_p),
                              ld, M, K, _p(h)))
    return h


def silu_grad(g: float) -> float:
    """silu'(g) in binary64."""
    return float(lib().orc_silu_grad(float(g)))


def silu_mul_bwd(gate, up, dh):
    """Backward of h = bf16(bf16(silu(gate)) * up): returns (dgate, dup) as bf16 bits [M,K].
    gate and up may be views of one [M, 2K] array (equal row strides); dh is dense [M,K]."""
    gate, up = np.asarray(gate), np.asarray(up)
    dh = _c(dh, np.uint16)
    if gate.dtype != np.uint16 or up.dtype != np.uint16 or gate.shape != up.shape or dh.shape != gate.shape:
        raise ValueError("gate, up and dh must be uint16 arrays of one shape")
    M, K = gate.shape
    if gate.strides != up.strides or gate.strides[1] != 2 or gate.strides[0] % 2:
        raise ValueError("gate and up need unit column stride and a common row stride")
    ld = gate.strides[0] // 2
    dgu = np.empty((M, 2 * K), np.uint16)
    dg, du = dgu[:, :K], dgu[:, K:]
    _check(lib().orc_silu_mul_bwd(gate.ctypes.data_as(ctypes.c_void_p), up.ctypes.data_as(ctypes.c_void_p), ld,
                                  _p(dh), M, K, dg.ctypes.data_as(ctypes.c_void_p),
                                  du.ctypes.data_as(ctypes.c_void_p), 2 * K))
    return dg, du


def rmsnorm_quant(x, gamma, eps):
    """RMSNorm, then the 1x128 row quantizer on its bf16 output."""
    h = rmsnorm(x, gamma, eps)
    out = quant_act(h)
    out["h"] = h
    return out


def silu_mul_quant(gate, up):
    """SiLU(gate) * up, then the 1x128 row quantizer on its bf16 output."""
    h = silu_mul(gate, up)
    out = quant_act(h)
    out["h"] = h
    return out
