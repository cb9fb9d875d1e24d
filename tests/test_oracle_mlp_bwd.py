"""Pins of the oracle's element-wise backward of the MLP activation, h = bf16(bf16(silu(g)) * u)
(Sec. 4.1: gradients between operators stay bf16): closed forms, finite differences, the
binary64 autograd of torch over every finite bf16 gate value, and the exactness of the two
bf16 x bf16 products."""
import math
from fractions import Fraction

import numpy as np
import torch

import jet_inputs as ji
import oracle as orc
from test_oracle_fused import FINITE, f32, nearest_bf16


def _bits(v):
    return ji.f32_to_bf16_bits(np.asarray(v, np.float32))


def _bwd(g, u, dh):
    g, u, dh = (np.asarray(t, np.uint16).reshape(1, -1) for t in (g, u, dh))
    dg, du = orc.silu_mul_bwd(g, u, dh)
    return dg[0], du[0]


def test_derivative_closed_forms_and_shape():
    assert orc.silu_grad(0.0) == 0.5
    assert orc.silu_grad(50.0) == 1.0 and abs(orc.silu_grad(-50.0)) < 1e-19
    # silu'(g) + silu'(-g) = 1 (silu(g) - silu(-g) = g)
    for g in (0.1, 0.7, 1.2785, 2.4, 5.0, 11.0):
        assert abs(orc.silu_grad(g) + orc.silu_grad(-g) - 1.0) < 1e-14
    # the derivative changes sign exactly once, at the minimum of silu (-0.27846 at g = -1.2785)
    lo, hi = -2.0, -1.0
    assert orc.silu_grad(lo) < 0 < orc.silu_grad(hi)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if orc.silu_grad(mid) < 0 else (lo, mid)
    assert abs(lo + 1.2785) < 1e-4 and abs(lo / (1.0 + math.exp(-lo)) + 0.27846) < 1e-5
    grid = np.linspace(-30, 30, 60001)
    vals = np.array([orc.silu_grad(float(g)) for g in grid])
    assert np.all(vals[grid < lo - 1e-3] < 0) and np.all(vals[grid > hi + 1e-3] > 0)
    # its extrema: 1.0998 at g = 2.3994 and, by the identity above, -0.0998 at g = -2.3994
    assert abs(grid[vals.argmax()] - 2.3994) < 2e-3 and abs(vals.max() - 1.0998) < 1e-4
    assert abs(grid[vals.argmin()] + 2.3994) < 2e-3 and abs(vals.min() + 0.0998) < 1e-4
    # central differences of the forward function (in binary64)
    silu = lambda x: x / (1.0 + math.exp(-x))
    for g in np.linspace(-12, 12, 97):
        h = 1e-5
        assert abs(orc.silu_grad(float(g)) - (silu(g + h) - silu(g - h)) / (2 * h)) < 1e-9


def test_dgate_for_every_finite_gate_value_against_torch_binary64_autograd():
    """da = 1 (dh = 1, u = 1): dgate = bf16(silu'(g)) for all 65280 finite bf16 g, against torch's
    binary64 backward of silu rounded by an independent nearest-neighbour search."""
    g = torch.tensor(f32(FINITE).astype(np.float64), requires_grad=True)
    torch.nn.functional.silu(g).sum().backward()
    want = np.array([nearest_bf16(float(v)) for v in g.grad.numpy()], np.uint16)
    one = np.full(FINITE.shape, 0x3F80, np.uint16)
    dg, du = _bwd(FINITE, one, one)
    # a zero result: both signs of zero are the real value rounded (silu'(-inf side) -> -0 underflows)
    same = (dg == want) | (((dg | want) & 0x7FFF) == 0)
    assert same.all(), np.argwhere(~same)[:5]
    # dup = bf16(1 * a) = the forward activation itself
    a = np.array([orc.silu_bf16(int(b)) for b in FINITE[::97]], np.uint16)
    assert np.array_equal(du[::97], a)


def test_products_are_single_roundings_of_exact_values():
    rng = np.random.default_rng(3)
    n = 4000
    g = _bits(rng.standard_normal(n) * 3)
    u = _bits(rng.standard_normal(n) * 2)
    dh = _bits(rng.standard_normal(n) * 1e-3)
    dg, du = _bwd(g, u, dh)
    for i in range(0, n, 7):
        a = float(f32([orc.silu_bf16(int(g[i]))])[0])
        d, uu, gg = float(f32([dh[i]])[0]), float(f32([u[i]])[0]), float(f32([g[i]])[0])
        assert du[i] == nearest_bf16(float(Fraction(d) * Fraction(a)))            # exact product, rounded once
        da = float(f32([nearest_bf16(float(Fraction(d) * Fraction(uu)))])[0])
        want = nearest_bf16(da * orc.silu_grad(gg))
        assert dg[i] == want or ((dg[i] | want) & 0x7FFF) == 0


def test_special_values_and_strides():
    one, two, half = 0x3F80, 0x4000, 0x3F00
    # g = 0: a = 0, silu' = 1/2  ->  dup = 0 * dh, dgate = (dh * u) / 2
    dg, du = _bwd([0x0000], [two], [one])
    assert du[0] == 0x0000 and dg[0] == one
    # g = 40: a = 40, silu' = 1 -> dup = 40 dh, dgate = dh * u
    g40 = _bits([40.0])[0]
    dg, du = _bwd([g40], [half], [two])
    assert f32([du[0]])[0] == 80.0 and f32([dg[0]])[0] == 1.0
    # g = -40: a = -0 (tiny), silu' ~ -1.7e-16: gradients vanish but keep their sign
    gm = _bits([-40.0])[0]
    dg, du = _bwd([gm], [one], [one])
    assert abs(f32([du[0]])[0]) < 1e-15 and -1e-14 < f32([dg[0]])[0] < 0
    # the two halves of one [M, 2K] tensor, and a dense copy of them, give the same result
    M, K = 5, 256
    gu = ji.mlp_intermediate(M, K, 9)
    dh = ji.grads(M, K, 10)
    a = orc.silu_mul_bwd(gu[:, :K], gu[:, K:], dh)
    b = orc.silu_mul_bwd(np.ascontiguousarray(gu[:, :K]), np.ascontiguousarray(gu[:, K:]), dh)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_gradient_of_the_whole_operator_in_binary64():
    """Against finite differences of h(g, u) = silu(g) u: the bf16 results sit within the two
    roundings of the true gradient (relative 2^-7 on each factor)."""
    rng = np.random.default_rng(4)
    n = 2000
    g = _bits(rng.standard_normal(n) * 2)
    u = _bits(rng.standard_normal(n) * 2)
    dh = _bits(rng.standard_normal(n))
    dg, du = _bwd(g, u, dh)
    G, U, D = (f32(t).astype(np.float64) for t in (g, u, dh))
    silu = lambda x: x / (1.0 + np.exp(-x))
    h = 1e-6
    want_du = D * silu(G)
    want_dg = D * U * (silu(G + h) - silu(G - h)) / (2 * h)
    got_du, got_dg = f32(du).astype(np.float64), f32(dg).astype(np.float64)
    assert np.all(np.abs(got_du - want_du) <= 2.0 ** -6.9 * np.abs(want_du) + 1e-30)
    assert np.all(np.abs(got_dg - want_dg) <= 2.0 ** -6.9 * np.abs(D * U) * 1.1 + 1e-30)
