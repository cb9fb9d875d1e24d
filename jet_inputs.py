"""Seeded synthetic inputs for the block-scaled FP8 linear layer.

This module serves both the CPU oracle's tests and the GPU library's tests and
benchmark.  It holds NONE of the method's arithmetic (no quantization, no
scales, no GEMM): only random tensors with the shapes and value structure of
the workloads, as bf16 bit patterns in ``uint16`` numpy arrays, generated on the
host so that both sides see identical bits.

Workloads (synthetic stand-ins for the dense-transformer layers the paper
trains; no dataset or checkpoint is involved):
  * activations X [M,K]: iid N(0,1); ceil(1% of K) seeded channel indices are
    multiplied by 50 (outlier channels);
  * weights W [N,K]: iid N(0, std 0.02);
  * output gradients dY [M,N]: iid N(0, std 1e-3); a Bernoulli(0.005) mask of
    entries is replaced by 1e-3 * Student-t(nu=3) draws (heavy tail);
  * weight update: W <- bf16(float(W) + N(0, std 1e-4)).
"""
from __future__ import annotations

import math

import numpy as np

GROUP = 128

# (name, N = out features, K = in features) of one decoder layer's linears
LAYER_8B = (
    ("q_proj", 4096, 4096),
    ("k_proj", 1024, 4096),
    ("v_proj", 1024, 4096),
    ("o_proj", 4096, 4096),
    ("gate_proj", 14336, 4096),
    ("up_proj", 14336, 4096),
    ("down_proj", 4096, 14336),
)
LAYER_32B = (
    ("q_proj", 5120, 5120),
    ("k_proj", 1024, 5120),
    ("v_proj", 1024, 5120),
    ("o_proj", 5120, 5120),
    ("gate_proj", 27648, 5120),
    ("up_proj", 27648, 5120),
    ("down_proj", 5120, 27648),
)

TENSOR_X, TENSOR_W, TENSOR_DY, TENSOR_UPDATE, TENSOR_POS = 0, 1, 2, 3, 4


def seed_for(config: int, matrix_index: int, tensor_id: int) -> int:
    """Seed = 1000*config + 10*matrix_index + tensor_id."""
    return 1000 * config + 10 * matrix_index + tensor_id


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16 (ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_f32(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def activations(M: int, K: int, seed: int) -> np.ndarray:
    """X [M,K] bf16 bits: N(0,1) with ceil(0.01*K) channels scaled by 50."""
    rng = _rng(seed)
    x = _normal_f32(rng, (M, K), 1.0)
    n_out = int(math.ceil(0.01 * K))
    cols = _rng(seed + 500_000).permutation(K)[:n_out]
    x[:, cols] *= np.float32(50.0)
    return f32_to_bf16_bits(x)


def weights(N: int, K: int, seed: int) -> np.ndarray:
    """W [N,K] bf16 bits: N(0, std 0.02)."""
    return f32_to_bf16_bits(_normal_f32(_rng(seed), (N, K), 0.02))


def grads(M: int, N: int, seed: int) -> np.ndarray:
    """dY [M,N] bf16 bits: N(0, std 1e-3) with 0.5% Student-t(nu=3) entries."""
    rng = _rng(seed)
    g = _normal_f32(rng, (M, N), 1e-3)
    mask = rng.random(size=(M, N), dtype=np.float32) < np.float32(0.005)
    n_heavy = int(mask.sum())
    g[mask] = (rng.standard_t(3.0, size=n_heavy) * 1e-3).astype(np.float32)
    return f32_to_bf16_bits(g)


def norm_weight(K: int, seed: int) -> np.ndarray:
    """RMSNorm weight [K] bf16 bits: 1 + N(0, std 0.1)."""
    return f32_to_bf16_bits(np.float32(1.0) + _normal_f32(_rng(seed), (K,), 0.1))


def mlp_intermediate(M: int, K: int, seed: int) -> np.ndarray:
    """One [M,2K] bf16 array holding the gate (columns 0..K-1) and up (K..2K-1) projections of an
    MLP block: N(0, std 2) with 0.5% of the entries scaled by 8."""
    rng = _rng(seed)
    h = _normal_f32(rng, (M, 2 * K), 2.0)
    mask = rng.random(size=(M, 2 * K), dtype=np.float32) < np.float32(0.005)
    h[mask] *= np.float32(8.0)
    return f32_to_bf16_bits(h)


def weight_update(w_bits: np.ndarray, seed: int) -> np.ndarray:
    """Synthetic optimizer step on the bf16 master weights: W + N(0, std 1e-4)."""
    w = bf16_bits_to_f32(w_bits)
    w = w + _normal_f32(_rng(seed), w.shape, 1e-4)
    return f32_to_bf16_bits(w)


def row_positions(n_rows: int, M: int, seed: int) -> np.ndarray:
    """n_rows distinct seeded positions in [0, M), in random order."""
    return _rng(seed).permutation(M)[:n_rows].astype(np.int64)


def sample_rows(M: int, n: int, seed: int) -> np.ndarray:
    """Seeded random rows plus the tile-boundary rows {0,127,128,M-1} that exist."""
    fixed = [r for r in (0, 127, 128, M - 1) if 0 <= r < M]
    extra = _rng(seed).permutation(M)[: max(0, min(n, M))].tolist()
    return np.array(sorted(set(fixed + extra)), dtype=np.int64)
