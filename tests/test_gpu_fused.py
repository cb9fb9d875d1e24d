"""GPU parity of the fused producers (RMSNorm -> FP8, SiLU*up -> FP8; Sec. 4.2 / 4.3): the FP8
codes and scales must be bit-identical to the oracle's "operator in bf16, then row quantizer"."""
import numpy as np
import pytest
import torch

import jet_inputs as ji
import oracle as orc
from jet_testlib import dev_bf16, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jet():
    import paper_2601_14243_amd as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def _same(name, got, want):
    got, want = np.asarray(got), np.asarray(want)
    if got.dtype == np.float32:
        got, want = got.view(np.uint32), want.astype(np.float32).view(np.uint32)
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{name}: {len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}"


def test_silu_of_every_finite_bf16_value(jet):
    """All 65280 finite gate values (up = 1, one 128-group each so that the group's scale cannot
    hide a wrong bf16): decode(q) * s must reproduce bf16(silu(g)) wherever FP8 resolves it, and
    codes and scales must equal the oracle's everywhere."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    bits = bits[(bits & 0x7F80) != 0x7F80]
    n = len(bits)
    K = 128
    gate = np.zeros((n, K), np.uint16)
    gate[:, 0] = bits                                  # the rest of the group is +0: amax is |silu(g)|
    up = np.full((n, K), 0x3F80, np.uint16)
    want = orc.silu_mul_quant(gate, up)
    got = jet.silu_mul_quant(dev_bf16(gate), dev_bf16(up))
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])
    # amax = |silu(g)| exactly: the scale alone carries the bf16 result (S = |a| / 448)
    a = ji.bf16_bits_to_f32(np.array([orc.silu_bf16(int(b)) for b in bits], np.uint16))
    s = host(got["s_row"])[:, 0]
    nz = a != 0
    assert np.array_equal(s[nz], (np.abs(a[nz]) / np.float32(448.0)).astype(np.float32))


@pytest.mark.parametrize("M,K,fused", [(256, 1024, True), (1, 128, False), (3, 14336, True), (77, 384, False),
                                       (1000, 2048, True), (129, 27648, False)])
def test_silu_mul_quant(jet, M, K, fused):
    both = ji.mlp_intermediate(M, K, seed=900 + M + K)
    gate, up = both[:, :K], both[:, K:]
    want = orc.silu_mul_quant(gate, up)
    if fused:                                           # the two halves of one [M,2K] tensor: ld = 2K
        t = dev_bf16(both)
        got = jet.silu_mul_quant(t[:, :K], t[:, K:])
    else:
        got = jet.silu_mul_quant(dev_bf16(np.ascontiguousarray(gate)), dev_bf16(np.ascontiguousarray(up)))
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])


def test_silu_mul_quant_extreme_values(jet):
    """Gate values where binary32 exp overflows or silu underflows, huge and tiny up values."""
    K = 128
    g_vals = [0xC2B0, 0xC2B2, 0xC2C8, 0xC2D0, 0xC2DC, 0xC300, 0x42B2, 0x4300, 0x0001, 0x8001, 0x0080, 0x3F80,
              0xFF7F, 0x7F7F, 0xC1A0, 0x41A0]
    u_vals = [0x3F80, 0x7E00, 0x0100, 0xBF80, 0x4000, 0x3F00, 0x3F80, 0x0080, 0x3F80, 0x7000, 0x7000, 0x0001,
              0x0080, 0x0080, 0x5000, 0xD000]
    gate = np.zeros((len(g_vals), K), np.uint16)
    up = np.full((len(g_vals), K), 0x3F80, np.uint16)
    for i, (g, u) in enumerate(zip(g_vals, u_vals)):
        gate[i, :] = g
        gate[i, 1::2] = 0x3F00
        up[i, :] = u
    want = orc.silu_mul_quant(gate, up)
    got = jet.silu_mul_quant(dev_bf16(gate), dev_bf16(up))
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])


@pytest.mark.parametrize("M,K,eps", [(256, 1024, 1e-6), (1, 128, 1e-5), (5, 4096, 1e-6), (300, 5120, 1e-6),
                                     (64, 8192, 1e-5), (9, 12288, 0.0), (4, 32768, 1e-6), (17, 640, 0.03)])
def test_rmsnorm_quant(jet, M, K, eps):
    x = ji.activations(M, K, seed=700 + M + K)
    gamma = ji.norm_weight(K, seed=701 + K)
    want = orc.rmsnorm_quant(x, gamma, eps)
    got = jet.rmsnorm_quant(dev_bf16(x), dev_bf16(gamma.reshape(1, K)).reshape(K), eps)
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])


def test_rmsnorm_quant_many_rows_of_the_hidden_size(jet):
    """4096 rows of the 8B-class hidden size: every row has its own mean, so a wrong rounding of the
    mean, the root or the reciprocal would show in some row."""
    M, K = 4096, 4096
    x = ji.activations(M, K, seed=ji.seed_for(2, 0, ji.TENSOR_X) + 5)
    # rows of very different magnitude: scale row m by 2^((m % 41) - 20)
    xf = ji.bf16_bits_to_f32(x) * np.exp2((np.arange(M) % 41) - 20).astype(np.float32)[:, None]
    x = ji.f32_to_bf16_bits(xf)
    gamma = ji.norm_weight(K, seed=77)
    want = orc.rmsnorm_quant(x, gamma, 1e-6)
    got = jet.rmsnorm_quant(dev_bf16(x), dev_bf16(gamma.reshape(1, K)).reshape(K), 1e-6)
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])


def test_rmsnorm_quant_zero_rows_and_tiny_rows(jet):
    K = 256
    gamma = ji.norm_weight(K, seed=9)
    x = ji.activations(6, K, seed=10)
    x[1, :] = 0                                          # all zeros: h = 0, S = 1 (eps > 0)
    x[2, :] = 0x8000                                     # all -0
    x[3, :] = 0x0001                                     # smallest bf16 subnormals
    x[4, :128] = 0
    want = orc.rmsnorm_quant(x, gamma, 1e-6)
    got = jet.rmsnorm_quant(dev_bf16(x), dev_bf16(gamma.reshape(1, K)).reshape(K), 1e-6)
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])


def test_fused_producer_feeds_the_gemm_like_the_plain_quantizer(jet):
    """RMSNorm -> FP8 -> FProp gives the bytes of (stored bf16 h) -> jet_quant_act -> FProp."""
    M, N, K = 96, 256, 512
    x, gamma = ji.activations(M, K, seed=51), ji.norm_weight(K, seed=52)
    w = ji.weights(N, K, seed=53)
    qw, sw = jet.quant_weight(dev_bf16(w))
    fused = jet.rmsnorm_quant(dev_bf16(x), dev_bf16(gamma.reshape(1, K)).reshape(K), 1e-6)
    plain = jet.quant_act(dev_bf16(orc.rmsnorm(x, gamma, 1e-6)))
    y1 = jet.fp8_linear_fwd(fused["q_row"], fused["s_row"], qw, sw)
    y2 = jet.fp8_linear_fwd(plain["q_row"], plain["s_row"], qw, sw)
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))


# ------------------------------------------------------------ full sizes (8B class, M = 16384)

def test_rmsnorm_quant_full_size(jet):
    M, K = 16384, 4096
    x = ji.activations(M, K, seed=ji.seed_for(2, 0, ji.TENSOR_X))
    gamma = ji.norm_weight(K, seed=78)
    want = orc.rmsnorm_quant(x, gamma, 1e-6)
    got = jet.rmsnorm_quant(dev_bf16(x), dev_bf16(gamma.reshape(1, K)).reshape(K), 1e-6)
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])


def test_silu_mul_quant_full_size(jet):
    """The [16384, 2 x 14336] output of a fused gate/up projection, both halves read in place."""
    M, K = 16384, 14336
    both = ji.mlp_intermediate(M, K, seed=ji.seed_for(2, 4, ji.TENSOR_X))
    want = orc.silu_mul_quant(both[:, :K], both[:, K:])
    t = dev_bf16(both)
    got = jet.silu_mul_quant(t[:, :K], t[:, K:])
    _same("q_row", host(got["q_row"]), want["q_row"])
    _same("s_row", host(got["s_row"]), want["s_row"])
