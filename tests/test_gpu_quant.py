"""GPU parity of the quantizers: FP8 codes and scales must be bit-identical to the
oracle (Sec. 2.1 formula, Sec. 4.2 granularities)."""
import numpy as np
import pytest
import torch

import jet_inputs as ji
import oracle as orc
from jet_testlib import dev, dev_bf16, host

pytestmark = pytest.mark.gpu
G = 128


@pytest.fixture(scope="module")
def jet():
    import paper_2601_14243_amd as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def _cmp(name, got, want):
    got = np.asarray(got)
    if got.dtype == np.float32:
        got, want = got.view(np.uint32), np.asarray(want, np.float32).view(np.uint32)
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{name}: {len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}"


@pytest.mark.parametrize("M,K", [(256, 1024), (1, 128), (1, 4096), (3, 256), (17, 384), (200, 512), (129, 14336)])
def test_row_quant_bf16(jet, M, K):
    x = ji.activations(M, K, seed=ji.seed_for(0, 0, ji.TENSOR_X) + M)
    want = orc.quant_act(x)
    got = jet.quant_act(dev_bf16(x))
    _cmp("q_row", host(got["q_row"]), want["q_row"])
    _cmp("s_row", host(got["s_row"]), want["s_row"])


@pytest.mark.parametrize("M,K", [(256, 1024), (128, 128), (384, 256), (1024, 640)])
@pytest.mark.parametrize("mode", ["col", "dual"])
def test_col_and_dual_quant_bf16(jet, M, K, mode):
    x = ji.grads(M, K, seed=ji.seed_for(2, 0, ji.TENSOR_DY) + M + K)
    row = mode == "dual"
    want = orc.quant_act(x, row=row, col=True)
    got = jet.quant_act(dev_bf16(x), row=row, col=True)
    for k in want:
        _cmp(k, host(got[k]), want[k])


@pytest.mark.parametrize("M,K", [(256, 512), (384, 128)])
@pytest.mark.parametrize("mode", ["row", "col", "dual"])
def test_quant_from_fp8_saved_activation(jet, M, K, mode):
    x = ji.activations(M, K, seed=77 + M)
    first = orc.quant_act(x)
    row, col = mode in ("row", "dual"), mode in ("col", "dual")
    want = orc.quant_act(first["q_row"], first["s_row"], src=orc.SRC_FP8_ROW, row=row, col=col)
    got = jet.quant_act(dev(first["q_row"]), dev(first["s_row"]), row=row, col=col)
    for k in want:
        _cmp(k, host(got[k]), want[k])


def test_every_bf16_amax_and_special_values(jet):
    """All 32639 positive finite bf16 values as a group's amax (from 2^-133 up to
    3.39e38: subnormal scales, the IEEE fallback of the divider), signed zeros,
    all-zero groups."""
    h = np.arange(1, 0x7F80, dtype=np.uint16)
    rng = np.random.default_rng(5)
    a = orc.bf16_to_f32(h)
    x = rng.uniform(-1, 1, size=(h.size, G)).astype(np.float32) * a[:, None]
    xb = ji.f32_to_bf16_bits(x)
    xb[:, 9] = h
    xb[:, 10] = 0x8000          # -0.0
    xb[:, 11] = 0x0000
    xb[:, 12] = h | 0x8000
    extra = np.zeros((3, G), np.uint16)
    extra[1, :] = 0x8000        # a group of negative zeros
    extra[2, 5] = 0x0001        # smallest subnormal alone
    xb = np.concatenate([xb, extra])
    pad = (-xb.shape[0]) % 128
    xb = np.concatenate([xb, np.zeros((pad, G), np.uint16)])
    want = orc.quant_act(xb, row=True, col=True)
    got = jet.quant_act(dev_bf16(xb), row=True, col=True)
    for k in want:
        _cmp(k, host(got[k]), want[k])
    got_row = jet.quant_act(dev_bf16(xb))
    _cmp("row-only q", host(got_row["q_row"]), want["q_row"])
    _cmp("row-only s", host(got_row["s_row"]), want["s_row"])


def test_rounding_boundaries_through_the_quantizer(jet):
    """Groups with amax = 448 * 2^j have S = 2^j exactly, so x / S is exact and the
    codes probe the E4M3 rounding directly: every bf16 value of a binade range hits
    ties, near-ties and the subnormal range."""
    vals = np.arange(0x3000, 0x4400, dtype=np.uint16)       # bf16 from 2^-31.. up to 512
    vals = vals[orc.bf16_to_f32(vals) <= 448.0]
    vals = np.concatenate([vals, vals | 0x8000])
    n = (vals.size + 126) // 127
    xb = np.zeros((n, G), np.uint16)
    flat = np.zeros(n * 127, np.uint16)
    flat[: vals.size] = vals
    xb[:, 1:] = flat.reshape(n, 127)
    xb[:, 0] = 0x43E0                                        # 448.0
    pad = (-n) % 128
    xb = np.concatenate([xb, np.zeros((pad, G), np.uint16)])
    want = orc.quant_act(xb, row=True, col=True)
    assert np.all(want["s_row"][:n, 0] == 1.0)
    got = jet.quant_act(dev_bf16(xb), row=True, col=True)
    for k in want:
        _cmp(k, host(got[k]), want[k])


@pytest.mark.parametrize("N,K", [(1024, 1024), (128, 128), (384, 256), (256, 1152)])
@pytest.mark.parametrize("transposed", [False, True])
def test_weight_quant(jet, N, K, transposed):
    w = ji.weights(N, K, seed=ji.seed_for(0, 0, ji.TENSOR_W) + N)
    want = orc.quant_weight(w, transposed=transposed)
    got = jet.quant_weight(dev_bf16(w), transposed=transposed)
    for name, g, wv in zip(("q", "s", "qT", "sT"), got, want):
        _cmp(name, host(g), wv)


def test_weight_requant_after_update(jet):
    w = ji.weights(256, 384, seed=3)
    w2 = ji.weight_update(w, seed=4)
    assert not np.array_equal(w, w2)
    want = orc.quant_weight(w2, transposed=True)
    got = jet.quant_weight(dev_bf16(w2), transposed=True)
    for name, g, wv in zip(("q", "s", "qT", "sT"), got, want):
        _cmp(name, host(g), wv)


def test_same_call_twice_same_bytes(jet):
    x = dev_bf16(ji.activations(256, 512, seed=1))
    a = jet.quant_act(x, row=True, col=True)
    b = jet.quant_act(x, row=True, col=True)
    for k in a:
        assert torch.equal(a[k], b[k])


def test_hardware_convert_on_every_rounding_boundary(jet):
    """The binary32 -> E4M3 conversion inside the kernels, probed value by value: with an FP8
    source whose codes are 1.0 and whose per-row scales are the test values, a column group of
    128 rows holds 127 arbitrary binary32 values v and one anchor 448, so S = 1 and the code
    written for a row is the conversion of v itself.  Test values: for every binade from 2^-13
    to 2^8 and each of the 16 leading 4-bit mantissa patterns (3 E4M3 bits + the rounding bit),
    the 19 low mantissa bits at 0, 1, 2, just below / at / above the half, all ones, and 40
    random patterns; both signs; plus zeros, the smallest subnormals and 448 itself.  Compared
    with the oracle's encoder directly and with its quantizer on the same tensors."""
    rng = np.random.default_rng(20240607)
    lows = np.array([0, 1, 2, 0x3FFFF, 0x40000, 0x40001, 0x7FFFE, 0x7FFFF], np.uint32)
    vals = []
    for e in range(127 - 13, 127 + 9):
        for top in range(16):
            low = np.concatenate([lows, rng.integers(0, 1 << 19, 40, dtype=np.uint32)])
            vals.append((np.uint32(e) << np.uint32(23)) | (np.uint32(top) << np.uint32(19)) | low)
    u = np.concatenate(vals)
    u = u[u <= np.float32(448.0).view(np.uint32)]
    extra = np.array([0x00000000, 0x00000001, 0x007FFFFF, 0x00800000, 0x3A800000, 0x3A7FFFFF, 0x3A800001,
                      np.float32(448.0).view(np.uint32)], np.uint32)
    u = np.concatenate([u, extra])
    u = np.concatenate([u, u | np.uint32(0x80000000)])
    n = len(u)
    groups = (n + 126) // 127
    pad = groups * 127 - n
    v = np.concatenate([u, np.zeros(pad, np.uint32)]).view(np.float32).reshape(groups, 127)
    M, K = groups * 128, 128
    codes = np.full((M, K), 0x38, np.uint8)                     # 1.0
    scales = np.ones((M, 1), np.float32)
    scales.reshape(groups, 128)[:, 1:] = v
    codes.reshape(groups, 128, K)[:, 0, :] = 0x7E               # the anchor row of every group: 448 x 1.0
    want = orc.quant_act(codes, scales, src=orc.SRC_FP8_ROW, row=False, col=True)
    got = jet.quant_act(dev(codes), dev(scales), row=False, col=True)
    gq, gs = host(got["q_colT"]), host(got["s_colT"])
    assert np.all(gs == 1.0)
    _cmp("q_colT", gq, want["q_colT"])
    direct = orc.e4m3_encode(v.reshape(-1))                     # the encoder alone, value by value
    assert np.array_equal(gq[0].reshape(groups, 128)[:, 1:].reshape(-1), direct)
    assert np.all(gq == gq[0:1])                                # all 128 columns saw the same values


def test_hardware_convert_on_every_binary32_value_up_to_448(jet):
    """The same probe, exhaustively: every binary32 value v with 2^-11 <= |v| <= 448 (all 2^23
    mantissas, both signs, 20 binades: 3.3e8 values) is converted by the kernel and compared with
    the oracle's encoder.  A row's scale runs over all sign and mantissa patterns of one binade;
    the columns of that row hold the E4M3 codes of the powers of two 2^-9 .. 2^8, so that the
    kernel's one multiply decode(code) * scale produces the same mantissa in 18 binades, exactly;
    a second pass with the scales divided by 4 reaches 2^-10 and 2^-11 (below, everything rounds
    to zero; the probe above samples that range).  Row 0 of every 128 rows is the anchor 448."""
    exps = np.arange(-9, 9)
    pow_codes = np.array([(1 << (e + 9)) if e < -6 else ((e + 7) << 3) for e in exps], np.uint8)
    assert np.array_equal(orc.e4m3_decode(pow_codes), np.ldexp(np.float32(1), exps))
    col_of = np.arange(G) % len(exps)                            # column k holds 2^exps[k % 18]
    chunk = 1 << 21
    total = 0
    for scale_shift, cols in ((0, range(len(exps))), (-2, (0, 1))):
        for c0 in range(0, 1 << 24, chunk):
            pat = np.arange(c0, c0 + chunk, dtype=np.uint32)
            sbits = ((pat >> np.uint32(23)) << np.uint32(31)) | np.uint32((127 + scale_shift) << 23) | (pat & np.uint32(0x7FFFFF))
            sv = sbits.view(np.float32)
            groups = -(-chunk // 127)
            v = np.concatenate([sv, np.zeros(groups * 127 - chunk, np.float32)]).reshape(groups, 127)
            M = groups * 128
            scales = np.ones((groups, 128), np.float32)
            scales[:, 1:] = v
            codes = np.empty((groups, 128, G), np.uint8)
            codes[:] = pow_codes[col_of]
            # 2^8 * |s| must stay at or below the anchor: rows with |s| > 1.75 hold a zero in those columns
            big = np.abs(scales) * np.float32(2.0 ** -scale_shift) > np.float32(1.75)
            codes[np.ix_(*map(np.arange, big.shape), np.flatnonzero(exps[col_of] == 8))] = np.where(
                big[:, :, None], 0, pow_codes[-1]).astype(np.uint8)
            codes[:, 0, :] = 0x7E
            got = jet.quant_act(dev(codes.reshape(M, G)), dev(scales.reshape(M, 1)), row=False, col=True)
            gq, gs = host(got["q_colT"]), host(got["s_colT"])
            assert np.all(gs == 1.0)
            for k in cols:
                x = v * np.ldexp(np.float32(1), int(exps[k]))
                if exps[k] == 8:
                    x = np.where(np.abs(x) > 448, np.float32(0) * v, x)     # decode(0) * s keeps the sign of s
                want = orc.e4m3_encode(x.reshape(-1))
                have = gq[k].reshape(groups, 128)[:, 1:].reshape(-1)
                bad = np.flatnonzero(have != want)
                assert bad.size == 0, (f"2^{exps[k] + scale_shift} binade: {bad.size} values differ, first "
                                       f"{x.reshape(-1)[bad[0]]!r}: got {have[bad[0]]:#x} want {want[bad[0]]:#x}")
                total += chunk
            assert all(np.array_equal(gq[k], gq[k % len(exps)]) for k in range(len(exps), G))
    assert total == 20 * (1 << 24)


def test_every_pair_of_bf16_value_and_group_maximum(jet):
    """The code of a value depends only on the value and on the largest magnitude of its group.
    All 5.3e8 pairs (|x| <= amax) of finite bf16 magnitudes, every second one negative: each group
    holds one amax and 127 consecutive smaller magnitudes.  The row kernel sees the groups as rows;
    the tile kernel (dual mode) sees them as columns, and mixtures of them as rows.  Codes and scales
    must equal the oracle's in every byte -- the divider (reciprocal, two corrections, IEEE fallback)
    and the hardware convert are exercised on every operand pair the bf16 path can produce."""
    per = G - 1
    amax_bits = np.arange(1, 0x7F80, dtype=np.int64)
    n_groups = (amax_bits + per - 1) // per
    edges = np.searchsorted(np.cumsum(n_groups), np.arange(0, n_groups.sum(), 400_000))
    edges = np.unique(np.concatenate([edges, [amax_bits.size]]))
    sign = np.where(np.arange(per) % 2 == 1, 0x8000, 0).astype(np.uint16)
    pairs = 0
    for lo, hi in zip(edges[:-1], edges[1:]):
        a = np.repeat(amax_bits[lo:hi], n_groups[lo:hi])                      # amax of every group
        first = np.concatenate([np.arange(n) for n in n_groups[lo:hi]]) * per  # its first magnitude
        vals = first[:, None] + np.arange(per)[None, :]
        live = vals < a[:, None]
        pairs += int(live.sum())
        grp = np.zeros((-(-a.size // G) * G, G), np.uint16)                    # padded with all-zero groups
        grp[:a.size, 0] = a
        grp[:a.size, 1:] = np.where(live, vals, 0).astype(np.uint16) | sign
        want_row = orc.quant_act(grp)
        got = jet.quant_act(dev_bf16(grp))
        _cmp(f"q_row, amax bits {lo + 1}..{hi}", host(got["q_row"]), want_row["q_row"])
        _cmp(f"s_row, amax bits {lo + 1}..{hi}", host(got["s_row"]), want_row["s_row"])
        # the same groups as the columns of [B * 128, 128] blocks
        x = np.ascontiguousarray(grp.reshape(-1, G, G).transpose(0, 2, 1)).reshape(-1, G)
        want = orc.quant_act(x, row=True, col=True)
        got = jet.quant_act(dev_bf16(x), row=True, col=True)
        for k in want:
            _cmp(f"{k} (tile kernel), amax bits {lo + 1}..{hi}", host(got[k]), want[k])
        # the column groups of x are the rows of grp
        assert np.array_equal(host(got["q_colT"]).reshape(G, -1, G).transpose(1, 0, 2).reshape(-1, G), want_row["q_row"])
    assert pairs == int((amax_bits).sum())
