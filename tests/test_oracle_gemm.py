"""Pins for the oracle's GEMMs (Sec. 2.2 definitions on Sec. 4.2 operands)."""
from fractions import Fraction

import numpy as np
import pytest

import jet_inputs as ji
import oracle as orc

G = 128


def _deq_row(q, s):
    return orc.e4m3_decode(q).astype(np.float64) * np.repeat(s.astype(np.float64), G, axis=1)


def _deq_block(q, s):
    return orc.e4m3_decode(q).astype(np.float64) * np.kron(s.astype(np.float64), np.ones((G, G)))


def test_hand_worked_all_twos_times_all_halves():
    # K=128: every x = 2.0 -> S = 2/448, code 448; every w = 0.5 -> S = 0.5/448, code 448.
    # p = 128 * 448^2 = 25,690,112 (exact in fp32); Y = 128 * 2 * 0.5 = 128.
    x = np.full((1, G), 0x4000, np.uint16)          # bf16 2.0
    w = np.full((G, G), 0x3F00, np.uint16)          # bf16 0.5
    qa = orc.quant_act(x)
    qw, sw = orc.quant_weight(w)
    assert np.all(qa["q_row"] == 0x7E) and np.all(qw == 0x7E)
    r = orc.gemm(qa["q_row"], qa["s_row"], qw, sw)
    # s = fl(2/448)*fl(.5/448) is not exactly 1/448^2, so allow the fp32 rounding of s
    assert np.all(np.abs(r["acc"] - 128.0) <= 128.0 * 2.0 ** -22)
    assert np.all(r["out"] == 0x4300)               # bf16 128.0
    assert np.allclose(r["exact"], 128.0, rtol=2.0 ** -22)
    # no cancellation: sum s |a b| = sum |s p| = the result itself, 128 products of 448^2 each
    s = float(np.float32(qa["s_row"][0, 0]) * np.float32(sw[0, 0]))
    assert np.all(r["sum_abs_prod"] == 128 * 448.0 ** 2 * s) and np.all(r["sum_abs"] == r["sum_abs_prod"])
    assert np.allclose(r["sum_abs_prod"], 128.0, rtol=2.0 ** -22)
    # alternate the sign of x: the result cancels to 0, the measure stays 128
    x[0, 1::2] = 0xC000                             # bf16 -2.0
    qa = orc.quant_act(x)
    r = orc.gemm(qa["q_row"], qa["s_row"], qw, sw)
    assert np.all(r["exact"] == 0.0) and np.all(r["sum_abs"] == 0.0)
    assert np.all(r["sum_abs_prod"] == 128 * 448.0 ** 2 * s)


@pytest.mark.parametrize("jlo,jhi,fp32_exact", [(-3, 4, False), (0, 2, True)])
def test_lossless_integer_gemm_zero_tolerance(jlo, jhi, fp32_exact):
    """Groups whose amax is 448*2^j hold (E4M3 integers)*2^j: quantization is
    exact, S = 2^j, and the GEMM equals an int64 matrix product times powers of
    two -- checked with zero tolerance (all partial sums fit 24 bits)."""
    rng = np.random.default_rng(1)
    M, N, K = 24, 256, 384
    ints = np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16], np.int64)
    xi = rng.choice(ints, size=(M, K)) * rng.choice([-1, 1], size=(M, K))
    wi = rng.choice(ints, size=(N, K)) * rng.choice([-1, 1], size=(N, K))
    jx = rng.integers(jlo, jhi, size=(M, K // G))
    jw = rng.integers(jlo, jhi, size=(N // G, K // G)) - (1 if fp32_exact else 0)
    xi[:, ::G] = 448                                 # pin every group's amax
    for nb in range(N // G):
        for kb in range(K // G):
            wi[nb * G, kb * G] = 448
    x = xi * 2.0 ** np.repeat(jx, G, axis=1)
    w = wi * 2.0 ** np.kron(jw, np.ones((G, G), np.int64))
    xb, wb = ji.f32_to_bf16_bits(x.astype(np.float32)), ji.f32_to_bf16_bits(w.astype(np.float32))
    assert np.array_equal(orc.bf16_to_f32(xb).astype(np.float64), x)
    qa = orc.quant_act(xb)
    qw, sw = orc.quant_weight(wb)
    assert np.array_equal(qa["s_row"], (2.0 ** jx).astype(np.float32))
    assert np.array_equal(sw, (2.0 ** jw).astype(np.float32))
    assert np.array_equal(orc.e4m3_decode(qa["q_row"]).astype(np.int64), xi)
    assert np.array_equal(orc.e4m3_decode(qw).astype(np.int64), wi)
    want = x @ w.T                                   # exact in fp64: small integers * 2^j
    r = orc.gemm(qa["q_row"], qa["s_row"], qw, sw)
    assert np.array_equal(r["exact"], want)
    if fp32_exact:
        # with the scales confined to {1/2, 1, 2} every partial sum is a multiple of 1/2
        # below 2^23, so the fp32 reference order is exact as well
        assert np.max(np.abs(want)) < 2.0 ** 22
        assert np.array_equal(r["acc"].astype(np.float64), want)
        assert np.array_equal(r["out"], orc.bf16_rne(want.astype(np.float32)))


def _frac(v):
    return Fraction(float(v))


@pytest.mark.parametrize("K", [128, 256])
def test_brute_force_exact_rationals_tiny(K):
    M, N = 3, 128
    x = ji.activations(M, K, seed=41)
    w = ji.weights(N, K, seed=42)
    qa = orc.quant_act(x)
    qw, sw = orc.quant_weight(w)
    cols = np.array([0, 1, 63, 127], np.int64)
    r = orc.gemm(qa["q_row"], qa["s_row"], qw, sw, cols=cols)
    dx, dw = orc.e4m3_decode(qa["q_row"]), orc.e4m3_decode(qw)
    for i in range(M):
        for jj, j in enumerate(cols):
            tot = Fraction(0)
            tabs = Fraction(0)
            for g in range(K // G):
                p = sum(_frac(dx[i, k]) * _frac(dw[j, k]) for k in range(g * G, (g + 1) * G))
                s = _frac(np.float32(qa["s_row"][i, g]) * np.float32(sw[j // G, g]))
                tot += p * s
                tabs += abs(p * s)
            assert abs(Fraction(float(r["exact"][i, jj])) - tot) <= abs(tot) * Fraction(1, 2 ** 50)
            assert abs(float(r["sum_abs"][i, jj]) - float(tabs)) <= float(tabs) * 1e-12
            # fp32 reference order stays within its own rounding-error bound of the truth
            sabs_elem = sum(abs(_frac(dx[i, k]) * _frac(dw[j, k])) *
                            _frac(np.float32(qa["s_row"][i, k // G]) * np.float32(sw[j // G, k // G]))
                            for k in range(K))
            bound = float(sabs_elem) * (G + K // G) * 2.0 ** -24
            assert abs(float(r["acc"][i, jj]) - float(tot)) <= bound
            # sum_g s_g sum_r |a_r b_r| (the cancellation measure of the GPU acceptance rule)
            assert abs(float(r["sum_abs_prod"][i, jj]) - float(sabs_elem)) <= float(sabs_elem) * 1e-12
            assert float(r["sum_abs_prod"][i, jj]) >= float(r["sum_abs"][i, jj]) * (1 - 1e-12)


def test_three_gemms_against_fp64_dequantised_matmul():
    """Non-square shapes; each GEMM kind against numpy's fp64 matmul of the
    dequantised operands (a transposed operand or a wrong scale index fails)."""
    M, N, K = 256, 384, 512
    x, w, dy = ji.activations(M, K, 51), ji.weights(N, K, 52), ji.grads(M, N, 53)
    qx = orc.quant_act(x, row=True, col=True)
    qdy = orc.quant_act(dy, row=True, col=True)
    qw, sw, qwT, swT = orc.quant_weight(w, transposed=True)
    X, W, DY = _deq_row(qx["q_row"], qx["s_row"]), _deq_block(qw, sw), _deq_row(qdy["q_row"], qdy["s_row"])
    XT, DYT = _deq_row(qx["q_colT"], qx["s_colT"]), _deq_row(qdy["q_colT"], qdy["s_colT"])

    acc, y = orc.fp8_linear_fwd(qx["q_row"], qx["s_row"], qw, sw)
    ref = X @ W.T
    assert acc.shape == (M, N)
    assert np.max(np.abs(acc - ref)) <= 1e-5 * np.max(np.abs(ref))
    assert np.array_equal(y, orc.bf16_rne(acc))

    acc, dx = orc.fp8_linear_dgrad(qdy["q_row"], qdy["s_row"], qwT, swT)
    ref = DY @ W
    assert acc.shape == (M, K)
    assert np.max(np.abs(acc - ref)) <= 1e-5 * np.max(np.abs(ref))

    acc, dw = orc.fp8_linear_wgrad(qdy["q_colT"], qdy["s_colT"], qx["q_colT"], qx["s_colT"])
    ref = DYT @ XT.T                                  # [N,M] x [M,K]
    assert acc.shape == (N, K)
    assert np.max(np.abs(acc - ref)) <= 1e-5 * np.max(np.abs(ref))

    # exact companion agrees with fp64 to fp64 accuracy
    r = orc.gemm(qx["q_row"], qx["s_row"], qw, sw, rows=np.arange(0, M, 37), cols=np.arange(0, N, 29))
    # (s is the fp32-rounded product of the two scales, the dequantised operands carry
    #  the unrounded one: 2^-24 relative)
    ref = (X @ W.T)[np.ix_(np.arange(0, M, 37), np.arange(0, N, 29))]
    assert np.all(np.abs(r["exact"] - ref) <= 2.0 ** -23 * r["sum_abs"])


def test_quantised_layer_tracks_the_unquantised_one():
    """Sanity band (not parity): against fp64 products of the bf16 inputs the
    relative Frobenius error of all three GEMMs is a few percent, which also
    fixes WHAT each GEMM computes (Sec. 2.2): Y = X W^T, dX = dY W, dW = dY^T X."""
    M, N, K = 256, 256, 384
    x, w, dy = ji.activations(M, K, 61), ji.weights(N, K, 62), ji.grads(M, N, 63)
    X, W, DY = (orc.bf16_to_f32(t).astype(np.float64) for t in (x, w, dy))
    qx = orc.quant_act(x, row=True, col=True)
    qdy = orc.quant_act(dy, row=True, col=True)
    qw, sw, qwT, swT = orc.quant_weight(w, transposed=True)

    def rel(a, b):
        return np.linalg.norm(a - b) / np.linalg.norm(b)

    acc, _ = orc.fp8_linear_fwd(qx["q_row"], qx["s_row"], qw, sw)
    assert rel(acc, X @ W.T) < 0.05
    acc, _ = orc.fp8_linear_dgrad(qdy["q_row"], qdy["s_row"], qwT, swT)
    assert rel(acc, DY @ W) < 0.05
    acc, _ = orc.fp8_linear_wgrad(qdy["q_colT"], qdy["s_colT"], qx["q_colT"], qx["s_colT"])
    assert rel(acc, DY.T @ X) < 0.05


def test_reference_order_within_bound_of_exact():
    M, N, K = 32, 128, 1024
    x, w = ji.activations(M, K, 71), ji.weights(N, K, 72)
    qa = orc.quant_act(x)
    qw, sw = orc.quant_weight(w)
    r = orc.gemm(qa["q_row"], qa["s_row"], qw, sw)
    bound = (G + K // G) * 2.0 ** -24 * r["sum_abs"] * 16   # sum_abs uses |p|, not sum|a b|: slack
    assert np.all(np.abs(r["acc"] - r["exact"]) <= bound + 1e-30)


def test_linearity_under_power_of_two_and_row_permutation():
    M, N, K = 16, 128, 256
    x, w = ji.activations(M, K, 81), ji.weights(N, K, 82)
    qa = orc.quant_act(x)
    qw, sw = orc.quant_weight(w)
    base = orc.gemm(qa["q_row"], qa["s_row"], qw, sw)["acc"]
    x2 = ji.f32_to_bf16_bits(orc.bf16_to_f32(x) * np.float32(8.0))
    qa2 = orc.quant_act(x2)
    assert np.array_equal(orc.gemm(qa2["q_row"], qa2["s_row"], qw, sw)["acc"], base * np.float32(8.0))
    perm = np.random.default_rng(5).permutation(M)
    qp = orc.quant_act(x[perm])
    got = orc.gemm(qp["q_row"], qp["s_row"], qw, sw)["acc"]
    assert np.array_equal(got.view(np.uint32), base[perm].view(np.uint32))
    # a row computed alone equals the same row inside the larger call
    one = orc.gemm(qa["q_row"][3:4], qa["s_row"][3:4], qw, sw)["acc"]
    assert np.array_equal(one.view(np.uint32), base[3:4].view(np.uint32))


def test_sampling_matches_full():
    M, N, K = 40, 256, 256
    x, w = ji.activations(M, K, 91), ji.weights(N, K, 92)
    qa = orc.quant_act(x)
    qw, sw = orc.quant_weight(w)
    full = orc.gemm(qa["q_row"], qa["s_row"], qw, sw)
    rows, cols = np.array([39, 0, 17]), np.array([255, 128, 127, 3])
    part = orc.gemm(qa["q_row"], qa["s_row"], qw, sw, rows=rows, cols=cols)
    for k in ("acc", "out", "exact", "sum_abs", "sum_abs_prod"):
        assert np.array_equal(part[k], full[k][np.ix_(rows, cols)])


def test_row_scale_mode_uses_per_row_scales():
    # WGrad mode: scaling one row of the second operand's scales by 2 scales one output column
    N, K, M = 128, 128, 256
    dy, x = ji.grads(M, N, 95), ji.activations(M, K, 96)
    a, b = orc.quant_act(dy, row=False, col=True), orc.quant_act(x, row=False, col=True)
    base = orc.gemm(a["q_colT"], a["s_colT"], b["q_colT"], b["s_colT"], sb_mode=orc.SB_ROW)["acc"]
    sb = b["s_colT"].copy()
    sb[7, :] *= 2
    got = orc.gemm(a["q_colT"], a["s_colT"], b["q_colT"], sb, sb_mode=orc.SB_ROW)["acc"]
    want = base.copy()
    want[:, 7] *= 2
    assert np.array_equal(got, want)
