"""Pins for the oracle's number formats: E4M3 encode/decode and bf16 rounding.

None of these re-types the oracle's own formulas: they compare it with a
hand-worked table, with exhaustive structural properties of the 256 codes, and
with torch's independent CPU float8_e4m3fn / bfloat16 conversions.
"""
import os

import numpy as np
import pytest
import torch

import oracle as orc


def _hand_table(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "e4m3_hand_table.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            val, code = line.split()[:2]
            rows.append((np.float32(float(val)), int(code, 16)))
    return rows


def test_hand_table(golden_dir):
    rows = _hand_table(golden_dir)
    assert len(rows) >= 30
    vals = np.array([r[0] for r in rows], np.float32)
    want = np.array([r[1] for r in rows], np.uint8)
    got = orc.e4m3_encode(vals)
    bad = [(float(v), hex(w), hex(g)) for v, w, g in zip(vals, want, got) if w != g]
    assert not bad, bad


def test_delta_max_is_448():
    # Sec. 2.1: the largest representable E4M3 value is 448.
    dec = orc.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert np.nanmax(dec) == 448.0 and np.nanmin(dec) == -448.0
    assert dec[0x7E] == 448.0


def test_all_256_codes_structure():
    codes = np.arange(256, dtype=np.uint8)
    dec = orc.e4m3_decode(codes)
    nan = np.isnan(dec)
    assert list(codes[nan]) == [0x7F, 0xFF]           # the only NaNs; no infinities
    assert not np.isinf(dec).any()
    pos = dec[0:0x7F]
    assert pos[0] == 0.0 and (np.diff(pos) > 0).all()  # strictly monotone in the code
    neg = dec[0x80:0xFF]
    assert np.array_equal(neg, -pos) and np.signbit(neg[0])
    # round trip of every non-NaN code
    rt = orc.e4m3_encode(dec[~nan])
    assert np.array_equal(rt, codes[~nan])
    # spacing: 8 codes per binade, quantum 2^-9 below 2^-6
    assert pos[1] == 2.0 ** -9 and pos[8] == 2.0 ** -6
    assert np.allclose(np.diff(pos[:9]), 2.0 ** -9, rtol=0, atol=0)
    for e in range(1, 15):
        blk = pos[8 * e: 8 * e + 8]
        assert blk[0] == 2.0 ** (e - 7)
        assert np.all(np.diff(blk) == 2.0 ** (e - 10))


def test_decode_matches_torch_float8():
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).float().numpy()
    dec = orc.e4m3_decode(codes.numpy())
    assert np.array_equal(np.isnan(ref), np.isnan(dec))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok].view(np.uint32), dec[ok].view(np.uint32))


def test_midpoints_go_to_even_and_neighbours_to_nearest():
    pos = orc.e4m3_decode(np.arange(0x7F, dtype=np.uint8)).astype(np.float64)
    for c in range(0x7E):
        lo, hi = pos[c], pos[c + 1]
        mid = np.float32((lo + hi) / 2)          # exact in fp32
        assert float(mid) == (lo + hi) / 2
        even = c if c % 2 == 0 else c + 1
        assert orc.e4m3_encode(mid)[()] == even, (c, mid)
        below = np.nextafter(mid, np.float32(0))
        above = np.nextafter(mid, np.float32(1e9))
        assert orc.e4m3_encode(below)[()] == c
        assert orc.e4m3_encode(above)[()] == c + 1
        assert orc.e4m3_encode(-mid)[()] == (even | 0x80)


def test_encode_matches_torch_float8_in_range():
    # torch's CPU conversion is an independent RNE implementation; it differs
    # only beyond the saturation threshold (it yields NaN where the oracle
    # saturates), so compare on |t| <= 464.
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 2 ** 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    t = bits.view(np.float32)
    t = t[np.isfinite(t) & (np.abs(t) <= 464.0)]
    # add a dense sweep of the interesting range and tiny values
    dense = np.concatenate([
        np.linspace(-464, 464, 400_001, dtype=np.float32),
        (rng.standard_normal(400_000) * 0.02).astype(np.float32),
        (rng.standard_normal(400_000) * 2.0 ** -8).astype(np.float32),
    ])
    t = np.concatenate([t, dense])
    ref = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = orc.e4m3_encode(t)
    assert np.array_equal(ref, got)


def test_saturation_never_nan():
    t = np.array([464.0, 464.0001, 480, 1e4, 3e38, np.inf], np.float32)
    assert np.all(orc.e4m3_encode(t) == 0x7E)
    assert np.all(orc.e4m3_encode(-t) == 0xFE)


def test_bf16_rne_matches_torch():
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 2 ** 32, size=1_000_000, dtype=np.uint64).astype(np.uint32)
    v = bits.view(np.float32)
    v = v[np.isfinite(v)]
    # exact ties and near ties
    base = (bits[:100_000] & np.uint32(0xFFFF0000)) | np.uint32(0x8000)
    ties = base.view(np.float32)
    ties = ties[np.isfinite(ties)]
    v = np.concatenate([v, ties, np.nextafter(ties, np.float32(0)), np.array([0.0, -0.0, 1.0, 3.3895314e38], np.float32)])
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = orc.bf16_rne(v)
    assert np.array_equal(ref, got)


def test_bf16_hand_cases():
    # 1 + 2^-8 is halfway between 1.0 (even) and 1 + 2^-7 -> 1.0
    assert orc.bf16_rne(np.float32(1 + 2.0 ** -8))[()] == 0x3F80
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd) and 1+2^-6 (even) -> 1+2^-6
    assert orc.bf16_rne(np.float32(1 + 3 * 2.0 ** -8))[()] == 0x3F82
    assert orc.bf16_rne(np.float32(-2.5))[()] == 0xC020
