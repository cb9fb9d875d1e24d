"""The MLP block with FP8-saved activations, forward and backward (Sec. 4.1, Sec. 4.2): the
element-wise backward kernel bit for bit against the oracle, then the whole block stage by stage
(every stage's GPU output against the oracle run on that stage's GPU inputs), end to end against
the oracle's own composition, and against binary64 autograd of the unquantized block."""
import numpy as np
import pytest
import torch

import jet_inputs as ji
import oracle as orc
from jet_testlib import check_gemm, dev_bf16, host, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jet():
    import paper_2601_14243_amd as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def _same(name, got, want):
    bad = np.argwhere(np.asarray(got) != np.asarray(want))
    assert bad.size == 0, f"{name}: {len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]:#x} want {want[tuple(bad[0])]:#x}"


def _same_or_zero(name, got, want):
    """bf16 bit patterns equal; where the result is a zero its sign is not compared (a real value of
    magnitude below the bf16 range rounds to a zero of either sign consistently on both sides, but a
    product that underflows in binary32 on one side may differ)."""
    got, want = np.asarray(got), np.asarray(want)
    bad = np.argwhere((got != want) & (((got | want) & 0x7FFF) != 0))
    assert bad.size == 0, f"{name}: {len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]:#x} want {want[tuple(bad[0])]:#x}"


def test_silu_mul_bwd_every_gate_value(jet):
    """Every bf16 gate value of magnitude below 2^64 (beyond, dh * silu(g) leaves the binary32 range,
    which the operator's contract excludes) against several (dh, u): dgate and dup bit for bit."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    bits = bits[((bits >> 7) & 0xFF) < 127 + 64]
    n = len(bits)
    K = 128
    rng = np.random.default_rng(11)
    gate = np.tile(bits[:, None], (1, K))
    up = ji.f32_to_bf16_bits(rng.standard_normal((n, K)).astype(np.float32) * 2)
    dh = ji.f32_to_bf16_bits(rng.standard_normal((n, K)).astype(np.float32) * np.float32(2.0) ** rng.integers(-12, 3, (n, K)))
    up[:, 0], dh[:, 0] = 0x3F80, 0x3F80                   # (1, 1): dgate = bf16(silu'(g)) itself
    up[:, 1], dh[:, 1] = 0xBF80, 0x3F80
    want_g, want_u = orc.silu_mul_bwd(gate, up, dh)
    got = host_bits(jet.silu_mul_bwd(dev_bf16(gate), dev_bf16(up), dev_bf16(dh)))
    _same("dup", got[:, K:], want_u)
    _same_or_zero("dgate", got[:, :K], want_g)


@pytest.mark.parametrize("M,K,fused", [(256, 1024, True), (1, 128, False), (77, 384, True), (513, 3584, True)])
def test_silu_mul_bwd_shapes_and_strides(jet, M, K, fused):
    both = ji.mlp_intermediate(M, K, seed=1200 + M + K)
    dh = ji.grads(M, K, seed=1300 + M)
    want_g, want_u = orc.silu_mul_bwd(both[:, :K], both[:, K:], dh)
    if fused:
        t = dev_bf16(both)
        got = jet.silu_mul_bwd(t[:, :K], t[:, K:], dev_bf16(dh))
    else:
        got = jet.silu_mul_bwd(dev_bf16(np.ascontiguousarray(both[:, :K])), dev_bf16(np.ascontiguousarray(both[:, K:])), dev_bf16(dh))
    got = host_bits(got)
    _same("dup", got[:, K:], want_u)
    _same_or_zero("dgate", got[:, :K], want_g)


def _oracle_block(x, w_gu, w_d, dy, I):
    """The block in the oracle's own arithmetic, end to end (its GEMM results in reference order)."""
    qx = orc.quant_act(x)
    q_gu, s_gu, q_guT, s_guT = orc.quant_weight(w_gu, transposed=True)
    q_d, s_d, q_dT, s_dT = orc.quant_weight(w_d, transposed=True)
    gu = orc.fp8_linear_fwd(qx["q_row"], qx["s_row"], q_gu, s_gu)[1]
    qh = orc.silu_mul_quant(gu[:, :I], gu[:, I:])
    y = orc.fp8_linear_fwd(qh["q_row"], qh["s_row"], q_d, s_d)[1]
    qdy = orc.quant_act(dy, row=True, col=True)
    dh = orc.fp8_linear_dgrad(qdy["q_row"], qdy["s_row"], q_dT, s_dT)[1]
    qhT = orc.quant_act(qh["q_row"], qh["s_row"], src=orc.SRC_FP8_ROW, row=False, col=True)
    dw_d = orc.fp8_linear_wgrad(qdy["q_colT"], qdy["s_colT"], qhT["q_colT"], qhT["s_colT"])[1]
    dg, du = orc.silu_mul_bwd(gu[:, :I], gu[:, I:], dh)
    dgu = np.concatenate([dg, du], axis=1)
    qdgu = orc.quant_act(dgu, row=True, col=True)
    dx = orc.fp8_linear_dgrad(qdgu["q_row"], qdgu["s_row"], q_guT, s_guT)[1]
    qxT = orc.quant_act(qx["q_row"], qx["s_row"], src=orc.SRC_FP8_ROW, row=False, col=True)
    dw_gu = orc.fp8_linear_wgrad(qdgu["q_colT"], qdgu["s_colT"], qxT["q_colT"], qxT["s_colT"])[1]
    return {"y": y, "dx": dx, "dw_gu": dw_gu, "dw_d": dw_d}


def _rel(a_bits, b):
    a = ji.bf16_bits_to_f32(a_bits).astype(np.float64)
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def test_mlp_block_forward_and_backward(jet):
    from paper_2601_14243_amd import mlp_block
    M, H, I = 256, 512, 1024
    x = ji.activations(M, H, 1401)
    w_gu = ji.weights(2 * I, H, 1402)
    w_d = ji.weights(H, I, 1403)
    dy = ji.grads(M, H, 1404)
    # gate/up pre-activations of a unit-variance order so that SiLU is exercised away from 0
    w_gu = ji.f32_to_bf16_bits(ji.bf16_bits_to_f32(w_gu) * np.float32(2.0))

    W = mlp_block.MlpWeights(dev_bf16(w_gu), dev_bf16(w_d))
    y, saved = mlp_block.forward(dev_bf16(x), W)
    out = mlp_block.backward(saved, dev_bf16(dy), W)
    torch.cuda.synchronize()

    # ---- stage by stage: the oracle on the GPU's own inputs of each stage ----
    q_gu, s_gu, q_guT, s_guT = orc.quant_weight(w_gu, transposed=True)
    q_d, s_d, q_dT, s_dT = orc.quant_weight(w_d, transposed=True)
    for got, want, name in zip(W.gu + W.d, (q_gu, s_gu, q_guT, s_guT, q_d, s_d, q_dT, s_dT),
                               ("q_gu", "s_gu", "q_guT", "s_guT", "q_d", "s_d", "q_dT", "s_dT")):
        assert np.array_equal(host(got), want), name
    oqx = orc.quant_act(x)
    gqx, gqs = host(saved["qx"]["q_row"]), host(saved["qx"]["s_row"])
    assert np.array_equal(gqx, oqx["q_row"]) and np.array_equal(gqs, oqx["s_row"])
    gu = host_bits(saved["gu"])
    check_gemm(gu, orc.gemm(gqx, gqs, q_gu, s_gu), "block gate/up fprop", operands=(gqx, gqs, q_gu, s_gu, False))
    oqh = orc.silu_mul_quant(gu[:, :I], gu[:, I:])
    gqh, gsh = host(saved["qh"]["q_row"]), host(saved["qh"]["s_row"])
    assert np.array_equal(gqh, oqh["q_row"]) and np.array_equal(gsh, oqh["s_row"])
    check_gemm(host_bits(y), orc.gemm(gqh, gsh, q_d, s_d), "block down fprop", operands=(gqh, gsh, q_d, s_d, False))

    oqdy = orc.quant_act(dy, row=True, col=True)
    for k in ("q_row", "s_row", "q_colT", "s_colT"):
        assert np.array_equal(host(out["qdy"][k]), oqdy[k]), k
    dh = host_bits(out["dh"])
    check_gemm(dh, orc.gemm(oqdy["q_row"], oqdy["s_row"], q_dT, s_dT), "block down dgrad",
               operands=(oqdy["q_row"], oqdy["s_row"], q_dT, s_dT, False))
    oqhT = orc.quant_act(gqh, gsh, src=orc.SRC_FP8_ROW, row=False, col=True)
    assert np.array_equal(host(out["qhT"]["q_colT"]), oqhT["q_colT"]) and np.array_equal(host(out["qhT"]["s_colT"]), oqhT["s_colT"])
    check_gemm(host_bits(out["dw_d"]), orc.gemm(oqdy["q_colT"], oqdy["s_colT"], oqhT["q_colT"], oqhT["s_colT"], sb_mode=orc.SB_ROW),
               "block down wgrad", operands=(oqdy["q_colT"], oqdy["s_colT"], oqhT["q_colT"], oqhT["s_colT"], True))
    odg, odu = orc.silu_mul_bwd(gu[:, :I], gu[:, I:], dh)
    dgu = host_bits(out["dgu"])
    _same("dup", dgu[:, I:], odu)
    _same_or_zero("dgate", dgu[:, :I], odg)
    oqdgu = orc.quant_act(dgu, row=True, col=True)
    for k in ("q_row", "s_row", "q_colT", "s_colT"):
        assert np.array_equal(host(out["qdgu"][k]), oqdgu[k]), k
    check_gemm(host_bits(out["dx"]), orc.gemm(oqdgu["q_row"], oqdgu["s_row"], q_guT, s_guT), "block gate/up dgrad",
               operands=(oqdgu["q_row"], oqdgu["s_row"], q_guT, s_guT, False))
    oqxT = orc.quant_act(gqx, gqs, src=orc.SRC_FP8_ROW, row=False, col=True)
    assert np.array_equal(host(out["qxT"]["q_colT"]), oqxT["q_colT"]) and np.array_equal(host(out["qxT"]["s_colT"]), oqxT["s_colT"])
    check_gemm(host_bits(out["dw_gu"]), orc.gemm(oqdgu["q_colT"], oqdgu["s_colT"], oqxT["q_colT"], oqxT["s_colT"], sb_mode=orc.SB_ROW),
               "block gate/up wgrad", operands=(oqdgu["q_colT"], oqdgu["s_colT"], oqxT["q_colT"], oqxT["s_colT"], True))

    # ---- end to end against the oracle's own composition: the wiring is the same ----
    ob = _oracle_block(x, w_gu, w_d, dy, I)
    for k, g in (("y", y), ("dx", out["dx"]), ("dw_gu", out["dw_gu"]), ("dw_d", out["dw_d"])):
        r = _rel(host_bits(g), ji.bf16_bits_to_f32(ob[k]).astype(np.float64))
        print(f"block {k}: relative L2 distance GPU vs oracle composition {r:.2e}")
        assert r < 5e-3, (k, r)

    # ---- and against binary64 autograd of the unquantized block: WHAT is computed ----
    X = torch.tensor(ji.bf16_bits_to_f32(x).astype(np.float64), requires_grad=True)
    Wgu = torch.tensor(ji.bf16_bits_to_f32(w_gu).astype(np.float64), requires_grad=True)
    Wd = torch.tensor(ji.bf16_bits_to_f32(w_d).astype(np.float64), requires_grad=True)
    GU = X @ Wgu.T
    Y = (torch.nn.functional.silu(GU[:, :I]) * GU[:, I:]) @ Wd.T
    Y.backward(torch.tensor(ji.bf16_bits_to_f32(dy).astype(np.float64)))
    for k, g, want in (("y", y, Y.detach()), ("dx", out["dx"], X.grad), ("dw_gu", out["dw_gu"], Wgu.grad), ("dw_d", out["dw_d"], Wd.grad)):
        r = _rel(host_bits(g), want.numpy())
        print(f"block {k}: relative L2 distance FP8 block vs binary64 unquantized block {r:.3f}")
        assert r < 0.08, (k, r)

    sb = mlp_block.saved_bytes(M, H, I)
    assert sb["fp8_saved"] == saved["qx"]["q_row"].numel() + 4 * saved["qx"]["s_row"].numel() + 2 * saved["gu"].numel() \
        + saved["qh"]["q_row"].numel() + 4 * saved["qh"]["s_row"].numel()
