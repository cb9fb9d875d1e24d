"""Pins for the oracle's quantizers (Sec. 2.1 formula, Sec. 4.2 granularities)."""
import numpy as np
import pytest
import torch

import jet_inputs as ji
import oracle as orc

G = 128


def _all_positive_finite_bf16():
    h = np.arange(1, 0x7F80, dtype=np.uint16)       # subnormals .. largest finite
    return h, orc.bf16_to_f32(h)


def test_scale_sweep_all_bf16_amax():
    """Every positive finite bf16 as the group's amax: S = amax/448 > 0 and the
    amax element itself maps to the code of 448 (the formula maps max|X| onto
    Delta_max)."""
    h, a = _all_positive_finite_bf16()
    assert h.size == 32639
    x = np.zeros((h.size, G), np.uint16)
    x[:, 5] = h
    x[:, 77] = h | 0x8000                            # -amax as well
    out = orc.quant_act(x)
    S = out["s_row"][:, 0]
    want = (a.astype(np.float64) / 448.0)
    assert np.all(S > 0)
    # S is the fp32 nearest to amax/448: within half an ulp of the exact quotient
    ulp = np.spacing(S.astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(S.astype(np.float64) - want) <= 0.5 * ulp + 1e-300)
    assert np.all(out["q_row"][:, 5] == 0x7E)
    assert np.all(out["q_row"][:, 77] == 0xFE)
    others = np.delete(out["q_row"], [5, 77], axis=1)
    assert np.all(others == 0)


def test_zero_group_has_unit_scale_and_signed_zero_codes():
    x = np.zeros((2, 2 * G), np.uint16)
    x[0, 3] = 0x8000                                  # -0.0
    x[1, G + 1] = 0x3F80                              # 1.0 in the second group of row 1
    out = orc.quant_act(x)
    assert out["s_row"][0, 0] == 1.0 and out["s_row"][0, 1] == 1.0 and out["s_row"][1, 0] == 1.0
    assert out["q_row"][0, 3] == 0x80 and out["q_row"][0, 4] == 0x00
    assert out["s_row"][1, 1] == np.float32(1.0) / np.float32(448.0)
    assert out["q_row"][1, G + 1] == 0x7E


def test_every_nonzero_group_reaches_448_and_error_bound():
    x = ji.activations(64, 1024, seed=3)
    out = orc.quant_act(x, row=True, col=False)
    q, S = out["q_row"], out["s_row"]
    mag = (q & 0x7F).reshape(64, 8, G)
    assert np.all(mag.max(axis=2) == 0x7E)
    xf = orc.bf16_to_f32(x).astype(np.float64)
    deq = orc.e4m3_decode(q).astype(np.float64) * np.repeat(S, G, axis=1)
    Sx = np.repeat(S, G, axis=1).astype(np.float64)
    # half a quantum: 2^-4 relative in the normal range, 2^-10 * S absolute below it
    bound = np.maximum(2.0 ** -4 * np.abs(xf), 2.0 ** -10 * Sx) * (1 + 1e-6)
    assert np.all(np.abs(deq - xf) <= bound)


def test_matches_vectorised_numpy_plus_torch_float8():
    """Independent route: numpy fp32 amax / divisions on reshaped blocks, torch's
    float8 converter for the rounding.  Catches wrong group axes or indexing."""
    x = ji.activations(256, 512, seed=5)
    xf = orc.bf16_to_f32(x)
    out = orc.quant_act(x, row=True, col=True)
    # rows: groups along K
    blk = xf.reshape(256, 4, G)
    amax = np.abs(blk).max(axis=2)
    S = (amax / np.float32(448.0)).astype(np.float32)
    t = (blk / S[:, :, None]).astype(np.float32).reshape(256, 512)
    ref = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(out["s_row"], S)
    assert np.array_equal(out["q_row"], ref)
    # columns: groups along M, outputs transposed
    blk = xf.T.reshape(512, 2, G)
    amax = np.abs(blk).max(axis=2)
    S = (amax / np.float32(448.0)).astype(np.float32)
    t = (blk / S[:, :, None]).astype(np.float32).reshape(512, 256)
    ref = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(out["s_colT"], S)
    assert np.array_equal(out["q_colT"], ref)


def test_column_mode_equals_row_mode_on_transposed_input():
    x = ji.grads(256, 384, seed=9)
    col = orc.quant_act(x, row=False, col=True)
    row = orc.quant_act(np.ascontiguousarray(x.T), row=True, col=False)
    assert np.array_equal(col["q_colT"], row["q_row"])
    assert np.array_equal(col["s_colT"], row["s_row"])


@pytest.mark.parametrize("j", [-20, -3, 1, 7, 30])
def test_power_of_two_scaling_moves_only_the_scales(j):
    x = ji.activations(16, 256, seed=13)
    xf = orc.bf16_to_f32(x)
    x2 = ji.f32_to_bf16_bits(xf * np.float32(2.0 ** j))
    assert np.array_equal(orc.bf16_to_f32(x2), xf * np.float32(2.0 ** j))   # exact
    a, b = orc.quant_act(x), orc.quant_act(x2)
    assert np.array_equal(a["q_row"], b["q_row"])
    assert np.array_equal(b["s_row"], a["s_row"] * np.float32(2.0 ** j))


def test_idempotence_bf16_amax_sweep():
    """quantize(dequantize(quantize(x))) reproduces codes and scales: swept over
    every positive finite bf16 amax (the dequantised amax 448*S need not equal
    amax, but its scale must)."""
    h, a = _all_positive_finite_bf16()
    rng = np.random.default_rng(3)
    x = np.zeros((h.size, G), np.float32)
    x[:, :] = (rng.uniform(-1, 1, size=(h.size, G)).astype(np.float32)) * a[:, None]
    x[:, 17] = a
    xb = ji.f32_to_bf16_bits(x)
    first = orc.quant_act(xb)
    # the dequantised tensor enters the second pass through the FP8 source mode
    second = orc.quant_act(first["q_row"], first["s_row"], src=orc.SRC_FP8_ROW)
    assert np.array_equal(first["q_row"], second["q_row"])
    assert np.array_equal(first["s_row"], second["s_row"])


def test_fp8_source_column_mode_against_numpy():
    x = ji.activations(256, 256, seed=21)
    first = orc.quant_act(x)
    v = orc.e4m3_decode(first["q_row"]) * np.repeat(first["s_row"], G, axis=1)   # fp32 products
    assert v.dtype == np.float32
    out = orc.quant_act(first["q_row"], first["s_row"], src=orc.SRC_FP8_ROW, row=False, col=True)
    blk = v.T.reshape(256, 2, G)
    amax = np.abs(blk).max(axis=2)
    S = (amax / np.float32(448.0)).astype(np.float32)
    t = (blk / S[:, :, None]).astype(np.float32).reshape(256, 256)
    ref = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(out["s_colT"], S)
    assert np.array_equal(out["q_colT"], ref)


def test_weight_blocks_against_numpy_and_transpose_symmetry():
    w = ji.weights(384, 256, seed=31)
    q, s, qT, sT = orc.quant_weight(w, transposed=True)
    wf = orc.bf16_to_f32(w)
    blk = wf.reshape(3, G, 2, G)
    amax = np.abs(blk).max(axis=(1, 3))
    S = (amax / np.float32(448.0)).astype(np.float32)
    assert np.array_equal(s, S)
    t = (blk / S[:, None, :, None]).astype(np.float32).reshape(384, 256)
    ref = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(q, ref)
    # Sec. 4.2: the weight scheme is symmetric under transpose
    assert np.array_equal(qT, q.T) and np.array_equal(sT, s.T)
    q2, s2 = orc.quant_weight(np.ascontiguousarray(w.T))
    assert np.array_equal(q2, q.T) and np.array_equal(s2, s.T)


def test_tiny_amax_keeps_ieee_semantics():
    # amax so small that S is subnormal: no floor, no flush
    x = np.zeros((1, G), np.uint16)
    x[0, 0] = 0x0001            # smallest positive bf16 subnormal, 2^-133
    x[0, 1] = 0x0080            # 2^-126
    out = orc.quant_act(x)
    S = out["s_row"][0, 0]
    assert S == np.float32(2.0 ** -126) / np.float32(448.0) and S > 0
    assert out["q_row"][0, 1] == 0x7E
    assert out["q_row"][0, 0] == orc.e4m3_encode(np.float32(2.0 ** -133) / S)[()]


def test_rejects_bad_shapes_and_nonfinite():
    with pytest.raises(ValueError):
        orc.quant_act(np.zeros((4, 100), np.uint16))
    with pytest.raises(ValueError):
        orc.quant_act(np.zeros((100, 128), np.uint16), row=False, col=True)
    with pytest.raises(ValueError):
        orc.quant_weight(np.zeros((128, 64), np.uint16))
    bad = np.zeros((1, G), np.uint16)
    bad[0, 0] = 0x7F80          # +inf
    with pytest.raises(ValueError):
        orc.quant_act(bad)
