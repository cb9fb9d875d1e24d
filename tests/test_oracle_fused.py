"""Pins of the oracle's fused producers (RMSNorm and SiLU*up in bf16 module semantics, in
front of the 1x128 quantizer: Sec. 4.2 / 4.3) against closed forms, invariants, a binary64
numpy evaluation and torch's binary64 silu.  The quantizer behind them is pinned elsewhere."""
import math

import numpy as np
import pytest
import torch

import jet_inputs as ji
import oracle as orc

ALL_BF16 = np.arange(65536, dtype=np.uint32).astype(np.uint16)
FINITE = ALL_BF16[(ALL_BF16 & 0x7F80) != 0x7F80]


def f32(bits):
    return ji.bf16_bits_to_f32(np.asarray(bits, np.uint16))


def nearest_bf16(v: float) -> int:
    """Independent rounding of a Python float to bf16: search the three bf16 neighbours of
    the binary32 conversion and take the one nearest in exact rational arithmetic."""
    from fractions import Fraction
    if v == 0.0:
        return 0x8000 if math.copysign(1.0, v) < 0 else 0
    sign = 0x8000 if v < 0 else 0
    a = abs(v)
    base = int(np.float32(a).view(np.uint32)) >> 16
    best = None
    for cand in (base - 1, base, base + 1):
        if cand < 0 or cand > 0x7F80:
            continue
        cv = Fraction(float(f32([cand])[0])) if cand < 0x7F80 else Fraction(2) ** 128
        d = abs(cv - Fraction(a))
        key = (d, cand & 1)        # ties: even pattern
        if best is None or key < best[0]:
            best = (key, cand)
    return sign | best[1]


# ------------------------------------------------------------ double -> bf16

def test_bf16_from_double_matches_the_binary32_rounding_where_both_apply():
    rng = np.random.default_rng(5)
    vals = rng.standard_normal(2000).astype(np.float32) * np.float32(37.0)
    want = orc.bf16_rne(vals)
    got = np.array([orc.bf16_from_double(float(v)) for v in vals], np.uint16)
    assert np.array_equal(got, want)


def test_bf16_from_double_rounds_once():
    # 1 + 2^-8 is the tie between 1.0 and 1 + 2^-7; a hair above it must go up even though the
    # conversion to binary32 lands exactly on the tie (which would then go to the even 1.0)
    v = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(v) == np.float32(1.0 + 2.0 ** -8)
    assert orc.bf16_from_double(v) == 0x3F81
    assert orc.bf16_from_double(1.0 + 2.0 ** -8) == 0x3F80                 # the tie itself: even
    assert orc.bf16_from_double(1.0 + 2.0 ** -8 - 2.0 ** -40) == 0x3F80
    assert orc.bf16_from_double(1.0 + 3 * 2.0 ** -8) == 0x3F82             # tie between ..81 and ..82: even
    assert orc.bf16_from_double(-(1.0 + 2.0 ** -8 + 2.0 ** -40)) == 0xBF81


def test_bf16_from_double_subnormals_zero_and_overflow():
    assert orc.bf16_from_double(0.0) == 0x0000 and orc.bf16_from_double(-0.0) == 0x8000
    assert orc.bf16_from_double(2.0 ** -133) == 0x0001                     # smallest subnormal
    assert orc.bf16_from_double(2.0 ** -134) == 0x0000                     # tie with zero: even
    assert orc.bf16_from_double(2.0 ** -134 * 1.0001) == 0x0001
    assert orc.bf16_from_double(-3 * 2.0 ** -134) == 0x8002                # tie between 1 and 2 quanta: even
    assert orc.bf16_from_double(2.0 ** -126) == 0x0080                     # smallest normal
    big = float(f32([0x7F7F])[0])
    assert orc.bf16_from_double(big) == 0x7F7F
    assert orc.bf16_from_double(big * (1 + 2.0 ** -10)) == 0x7F7F
    assert orc.bf16_from_double(2.0 ** 128 * (1 - 2.0 ** -9)) == 0x7F80    # the tie with 2^128 goes to infinity
    for v in (0.1, -2.7, 1e-30, 3.3e38, 7.77e-40):
        assert orc.bf16_from_double(v) == nearest_bf16(v)


# ---------------------------------------------------------------------- silu

def test_silu_every_finite_bf16_input_against_torch_binary64():
    g = torch.from_numpy(f32(FINITE).astype(np.float64))
    ref = torch.nn.functional.silu(g).numpy()
    got = np.array([orc.silu_bf16(int(b)) for b in FINITE], np.uint16)
    want = np.array([nearest_bf16(float(v)) for v in ref], np.uint16)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, (hex(int(FINITE[bad[0]])), hex(int(got[bad[0]])), hex(int(want[bad[0]])))


def test_silu_closed_forms():
    assert orc.silu_bf16(0x0000) == 0x0000 and orc.silu_bf16(0x8000) == 0x8000     # silu(+-0) = +-0
    for bits in (0x4200, 0x4300, 0x4780, 0x7F7F):                                   # 32, 128, 65536, max: silu(g) = g
        assert orc.silu_bf16(bits) == bits
    assert orc.silu_bf16(0xC2DC) == 0x8000                                          # silu(-110) ~ -1.8e-46 -> -0
    assert orc.silu_bf16(0x3F80) == nearest_bf16(1.0 / (1.0 + math.exp(-1.0)))      # 0.7310585...
    assert orc.silu_bf16(0xBF80) == nearest_bf16(-1.0 / (1.0 + math.e))             # -0.2689414...
    # the minimum of silu is -0.27846... at g = -1.27846...
    vals = f32(np.array([orc.silu_bf16(int(b)) for b in FINITE], np.uint16))
    assert vals.min() == f32([nearest_bf16(-0.2784645427610738)])[0]
    at_min = f32(FINITE)[vals == vals.min()]
    assert at_min.min() > -1.5 and at_min.max() < -1.1 and at_min.min() <= -1.2784645 <= at_min.max()


def test_silu_symmetry_and_monotonicity():
    pos = FINITE[(FINITE & 0x8000) == 0]
    g = f32(pos).astype(np.float64)
    a_pos = f32(np.array([orc.silu_bf16(int(b)) for b in pos], np.uint16)).astype(np.float64)
    a_neg = f32(np.array([orc.silu_bf16(int(b) | 0x8000) for b in pos], np.uint16)).astype(np.float64)
    # silu(g) - silu(-g) = g, up to the two bf16 roundings
    tol = 2.0 ** -8 * (np.abs(a_pos) + np.abs(a_neg)) + 2.0 ** -133
    assert np.all(np.abs(a_pos - a_neg - g) <= tol)
    assert np.all(np.diff(a_pos) >= 0)                      # increasing on g >= 0 (pos is in increasing order)
    assert np.all(a_neg <= 0) and np.all(a_pos >= 0)


def test_silu_mul_is_the_bf16_product_and_honours_the_row_stride():
    M, K = 5, 256
    both = ji.mlp_intermediate(M, K, seed=11)
    gate, up = both[:, :K], both[:, K:]
    h = orc.silu_mul(gate, up)
    a = f32(np.array([[orc.silu_bf16(int(b)) for b in row] for row in gate], np.uint16))
    want = orc.bf16_rne((a * f32(up)).astype(np.float32))       # bf16 x bf16 is exact in binary32
    assert np.array_equal(h, want)
    assert np.array_equal(h, orc.silu_mul(np.ascontiguousarray(gate), np.ascontiguousarray(up)))
    out = orc.silu_mul_quant(gate, up)
    plain = orc.quant_act(h)
    assert np.array_equal(out["q_row"], plain["q_row"]) and np.array_equal(out["s_row"], plain["s_row"])


# ------------------------------------------------------------------- rmsnorm

def test_rmsnorm_one_hot_rows():
    # a single entry v in a row of K = 4096: mean = v^2/4096, r = 64/|v|, v r = +-64 up to 2^-23,
    # so h = +-64 gamma at that entry and (signed) zero elsewhere
    K = 4096
    gamma = ji.norm_weight(K, seed=3)
    x = np.zeros((6, K), np.uint16)
    vals = [0x3F80, 0xC0A0, 0x3DCD, 0x4479, 0xBF13, 0x2F80]    # 1, -5, 0.1, 996, -0.57, 2^-32
    cols = [0, 17, 127, 128, 2049, 4095]
    for m, (v, c) in enumerate(zip(vals, cols)):
        x[m, c] = v
    h = orc.rmsnorm(x, gamma, 0.0)
    for m, (v, c) in enumerate(zip(vals, cols)):
        sign = -1.0 if v & 0x8000 else 1.0
        assert f32(h[m, c:c + 1])[0] == np.float32(sign * 64.0) * f32(gamma[c:c + 1])[0]
        rest = np.delete(h[m], c)
        assert np.all((rest & 0x7FFF) == 0)


def test_rmsnorm_constant_rows_return_gamma():
    K = 384
    gamma = ji.norm_weight(K, seed=4)
    for bits in (0x3F80, 0x4049, 0xC2F7, 0x1F80, 0x5D80):       # 1, 3.14, -123.5, 2^-64, 2^60
        x = np.full((2, K), bits, np.uint16)
        h = orc.rmsnorm(x, gamma, 0.0)
        want = gamma ^ np.uint16(bits & 0x8000)
        assert np.array_equal(h[0], want) and np.array_equal(h[1], want)


def test_rmsnorm_eps_enters_under_the_root():
    # x = 2^-20 everywhere, eps = 2^-20: mean + eps = 2^-20 (1 + 2^-20), root = 2^-10 (1 + 2^-21),
    # x r = 2^-10 (1 - 2^-21 ...) -> bf16 2^-10; without eps the result would be gamma itself
    K = 256
    gamma = ji.norm_weight(K, seed=5)
    x = np.full((1, K), 0x3580, np.uint16)
    assert f32([0x3580])[0] == np.float32(2.0 ** -20)
    h = orc.rmsnorm(x, gamma, 2.0 ** -20)
    assert np.array_equal(f32(h[0]), f32(gamma) * np.float32(2.0 ** -10))


def test_rmsnorm_is_invariant_under_powers_of_two_when_eps_is_zero():
    M, K = 7, 640
    x = ji.activations(M, K, seed=21)
    gamma = ji.norm_weight(K, seed=22)
    h = orc.rmsnorm(x, gamma, 0.0)
    for e in (-20, -3, 5, 30):
        xs = ji.f32_to_bf16_bits(f32(x) * np.float32(2.0 ** e))
        assert np.array_equal(orc.rmsnorm(xs, gamma, 0.0), h)
    # and changes sign with x
    assert np.array_equal(orc.rmsnorm(x ^ np.uint16(0x8000), gamma, 0.0), h ^ np.uint16(0x8000))


@pytest.mark.parametrize("eps", [0.0, 1e-6, 1e-2, 10.0])
def test_rmsnorm_against_binary64_numpy(eps):
    M, K = 33, 1024
    x = ji.activations(M, K, seed=31)
    gamma = ji.norm_weight(K, seed=32)
    h = f32(orc.rmsnorm(x, gamma, eps)).astype(np.float64)
    xd, gd = f32(x).astype(np.float64), f32(gamma).astype(np.float64)
    ref = gd * xd / np.sqrt((xd * xd).mean(axis=1, keepdims=True) + float(np.float32(eps)))
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -126))) - 7)
    err = np.abs(h - ref) / ulp
    # two roundings to bf16: half an ulp of h, plus gamma x half an ulp of n, which is up to one ulp
    # of h when gamma n falls into the binade below n's; plus binary32 noise
    assert err.max() <= 1.51, err.max()
    assert np.median(err) < 0.35
    # the result is not the plain single rounding: that is what "bf16 module semantics" means
    single = f32(ji.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64)
    assert np.count_nonzero(single != h) > 0


def test_rmsnorm_quant_chains_the_row_quantizer():
    M, K = 9, 512
    x, gamma = ji.activations(M, K, seed=41), ji.norm_weight(K, seed=42)
    out = orc.rmsnorm_quant(x, gamma, 1e-6)
    plain = orc.quant_act(out["h"])
    assert np.array_equal(out["q_row"], plain["q_row"]) and np.array_equal(out["s_row"], plain["s_row"])


def test_fused_argument_errors():
    x, gamma = ji.activations(2, 128, seed=1), ji.norm_weight(128, seed=2)
    with pytest.raises(ValueError):
        orc.rmsnorm(x, gamma, -1.0)
    with pytest.raises(ValueError):
        orc.rmsnorm(x, gamma[:64], 1e-6)
    with pytest.raises(ValueError):
        orc.rmsnorm(np.zeros((1, 128), np.uint16), gamma, 0.0)       # 1/sqrt(0)
    with pytest.raises(ValueError):
        orc.rmsnorm(np.full((1, 128), 0x5F80, np.uint16), gamma, 0.0)    # mean of squares 2^128
    with pytest.raises(ValueError):
        orc.silu_mul(x, x[:, :64])
