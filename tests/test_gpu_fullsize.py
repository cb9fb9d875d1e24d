"""GPU parity at the full sizes of the workloads, in the launch configurations the
benchmark times (persistent 256x256 tile kernel, strip and skinny decode kernels).

The oracle cannot run a whole 10^12-MAC GEMM, so outputs are sampled: the oracle
quantizes the same seeded bf16 inputs (rows are independent for 1x128 row groups,
columns for 128x1 token groups) and computes the sampled output rows one by one;
the GPU computes everything and is compared on those rows element by element.
FP8 codes and scales: bit-exact.  GEMM outputs: the acceptance rule of
jet_testlib.check_gemm (2 bf16 ulp against the oracle's fp32 reference order on
at least 99.5 % of the elements, every element within the matrix core's
documented allowance of the exact value).

Row-level invariance between rollout-shaped and training-shaped calls (Sec. 4.1
of the paper: the inference graph is a subgraph of the training forward graph)
is checked on the real layer shapes across every forward kernel of the library.
"""
import numpy as np
import pytest
import torch

import jet_inputs as ji
import oracle as orc
from jet_testlib import DEV, check_gemm, dev_bf16, host, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jet():
    import paper_2601_14243_amd as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def _rows_of(t: torch.Tensor, rows: np.ndarray) -> np.ndarray:
    return host(t[torch.from_numpy(rows).to(t.device)])


def _rows_bits(t: torch.Tensor, rows: np.ndarray) -> np.ndarray:
    return host_bits(t[torch.from_numpy(rows).to(t.device)])


def _layer_case(jet, cfg, idx, layer, M, n_rows, do_fwd=True, do_dgrad=True, do_wgrad=True, wgrad_rows=()):
    """One linear of a layer at training size: quantizers in full where the oracle can
    afford it, GEMM outputs on sampled rows (all columns).  wgrad_rows: output rows of dW that
    are checked besides the seeded ones (rows on both sides of a launch seam)."""
    name, N, K = layer[idx]
    x = ji.activations(M, K, ji.seed_for(cfg, idx, ji.TENSOR_X))
    w = ji.weights(N, K, ji.seed_for(cfg, idx, ji.TENSOR_W))
    rows = ji.sample_rows(M, n_rows, ji.seed_for(cfg, idx, ji.TENSOR_POS))

    gw = jet.quant_weight(dev_bf16(w), transposed=True)
    oq, os_, oqT, osT = orc.quant_weight(w, transposed=True)
    assert np.array_equal(host(gw[0]), oq) and np.array_equal(host(gw[1]), os_), f"{name}: weight codes/scales"
    assert np.array_equal(host(gw[2]), oqT) and np.array_equal(host(gw[3]), osT), f"{name}: transposed copy"
    del w

    gx = jet.quant_act(dev_bf16(x))
    ox = orc.quant_act(x[rows])
    assert np.array_equal(_rows_of(gx["q_row"], rows), ox["q_row"]), f"{name}: X codes"
    assert np.array_equal(_rows_of(gx["s_row"], rows), ox["s_row"]), f"{name}: X scales"

    if do_fwd:
        y = jet.fp8_linear_fwd(gx["q_row"], gx["s_row"], gw[0], gw[1])
        ref = orc.gemm(ox["q_row"], ox["s_row"], oq, os_)
        check_gemm(_rows_bits(y, rows), ref, f"{name} fwd M={M}", operands=(ox["q_row"], ox["s_row"], oq, os_, False))
        del y

    if not (do_dgrad or do_wgrad):
        return
    dy = ji.grads(M, N, ji.seed_for(cfg, idx, ji.TENSOR_DY))
    gdy = jet.quant_act(dev_bf16(dy), row=True, col=True)
    if do_dgrad:
        ody = orc.quant_act(dy[rows])
        assert np.array_equal(_rows_of(gdy["q_row"], rows), ody["q_row"]), f"{name}: dY codes"
        assert np.array_equal(_rows_of(gdy["s_row"], rows), ody["s_row"]), f"{name}: dY scales"
        dx = jet.fp8_linear_dgrad(gdy["q_row"], gdy["s_row"], gw[2], gw[3])
        ref = orc.gemm(ody["q_row"], ody["s_row"], oqT, osT)
        check_gemm(_rows_bits(dx, rows), ref, f"{name} dgrad M={M}", operands=(ody["q_row"], ody["s_row"], oqT, osT, False))
        del dx

    if do_wgrad:
        # dW rows = output features n; the reduction runs over all M tokens
        nsel = ji.sample_rows(N, 6, ji.seed_for(cfg, idx, ji.TENSOR_POS) + 1)
        nsel = np.unique(np.concatenate([nsel, np.asarray(wgrad_rows, np.int64)])).astype(np.int64)
        ody_c = orc.quant_act(np.ascontiguousarray(dy[:, nsel]), row=False, col=True)
        assert np.array_equal(_rows_of(gdy["q_colT"], nsel), ody_c["q_colT"]), f"{name}: dY^T codes"
        assert np.array_equal(_rows_of(gdy["s_colT"], nsel), ody_c["s_colT"]), f"{name}: dY^T scales"
        # the FP8-saved X re-quantized along tokens, in full on both sides
        gxT = jet.quant_act(gx["q_row"], gx["s_row"], row=False, col=True)
        ox_full = orc.quant_act(x)
        oxT = orc.quant_act(ox_full["q_row"], ox_full["s_row"], src=orc.SRC_FP8_ROW, row=False, col=True)
        assert np.array_equal(host(gx["q_row"]), ox_full["q_row"]), f"{name}: X codes (all rows)"
        assert np.array_equal(host(gxT["q_colT"]), oxT["q_colT"]), f"{name}: X^T codes"
        assert np.array_equal(host(gxT["s_colT"]), oxT["s_colT"]), f"{name}: X^T scales"
        dw = jet.fp8_linear_wgrad(gdy["q_colT"], gdy["s_colT"], gxT["q_colT"], gxT["s_colT"])
        ref = orc.gemm(ody_c["q_colT"], ody_c["s_colT"], oxT["q_colT"], oxT["s_colT"], sb_mode=orc.SB_ROW)
        check_gemm(_rows_bits(dw, nsel), ref, f"{name} wgrad M={M}",
                   operands=(ody_c["q_colT"], ody_c["s_colT"], oxT["q_colT"], oxT["s_colT"], True))


# ---- config 2: training step of the 8B-class layer at M = 16384 ----

def test_8b_q_proj_training_step(jet):
    _layer_case(jet, 2, 0, ji.LAYER_8B, 16384, 24)


def test_8b_k_proj_training_step(jet):
    _layer_case(jet, 2, 1, ji.LAYER_8B, 16384, 24)


def test_8b_gate_proj_training_step(jet):
    # WGrad output 14336 x 4096 = 56 x 16 tiles of 256 x 256 = 3.5 rounds of 256 workgroups: output rows
    # from 12288 on are split off to the 128 x 128 tile kernel; rows on both sides of that seam
    _layer_case(jet, 2, 4, ji.LAYER_8B, 16384, 12, wgrad_rows=(0, 255, 12287, 12288, 12415, 12416, 14335))


def test_8b_down_proj_training_step(jet):
    # WGrad output 4096 x 14336 = 16 x 56 tiles: output columns from 12288 on are split off (the rows
    # checked span all columns, i.e. both launches and the row pitch of the partial launch);
    # DGrad reduces over N = 4096, output 16384 x 14336
    _layer_case(jet, 2, 6, ji.LAYER_8B, 16384, 10, wgrad_rows=(0, 127, 128, 4095))


# ---- config 4: 32B-class shapes ----

def test_32b_q_proj_forward_long_rollout(jet):
    _layer_case(jet, 4, 0, ji.LAYER_32B, 32768, 16, do_dgrad=False, do_wgrad=False)


def test_32b_k_proj_training_step_long_rollout(jet):
    _layer_case(jet, 4, 1, ji.LAYER_32B, 32768, 16)


def test_32b_gate_proj_training_step_long_rollout(jet):
    # the widest matrix of the configurations: DGrad reduces over N = 27648 (216 groups), WGrad over
    # 32768 tokens (256 groups) into a 27648 x 5120 output
    _layer_case(jet, 4, 4, ji.LAYER_32B, 32768, 6, wgrad_rows=(0, 27647))


def test_32b_down_proj_forward_long_rollout(jet):
    # the longest reduction of the configurations: K = 27648 (216 groups), X is 1.8 GB of bf16
    _layer_case(jet, 4, 6, ji.LAYER_32B, 32768, 6, do_dgrad=False, do_wgrad=False)


@pytest.mark.parametrize("idx", [0, 6])           # q_proj 5120x5120, down_proj 5120x27648
@pytest.mark.parametrize("M", [1, 64, 256])
def test_32b_decode(jet, idx, M):
    name, N, K = ji.LAYER_32B[idx]
    x = ji.activations(M, K, ji.seed_for(4, idx, ji.TENSOR_X) + M)
    w = ji.weights(N, K, ji.seed_for(4, idx, ji.TENSOR_W))
    gq, gs = jet.quant_weight(dev_bf16(w))
    oq, os_ = orc.quant_weight(w)
    gx = jet.quant_act(dev_bf16(x))
    ox = orc.quant_act(x)
    assert np.array_equal(host(gx["q_row"]), ox["q_row"]) and np.array_equal(host(gx["s_row"]), ox["s_row"])
    y = jet.fp8_linear_fwd(gx["q_row"], gx["s_row"], gq, gs)
    rows = ji.sample_rows(M, 8, 77 + M)
    ref = orc.gemm(ox["q_row"], ox["s_row"], oq, os_, rows=rows)
    check_gemm(host_bits(y)[rows], ref, f"32B {name} decode M={M}", operands=(ox["q_row"][rows], ox["s_row"][rows], oq, os_, False))


# ---- config 1: rollout decode shapes of the 8B-class layer ----

@pytest.mark.parametrize("idx", [0, 1, 4, 6])     # q, k, gate, down
@pytest.mark.parametrize("M", [1, 8, 32, 128])
def test_8b_decode(jet, idx, M):
    name, N, K = ji.LAYER_8B[idx]
    x = ji.activations(M, K, ji.seed_for(1, idx, ji.TENSOR_X) + M)
    w = ji.weights(N, K, ji.seed_for(1, idx, ji.TENSOR_W))
    gq, gs = jet.quant_weight(dev_bf16(w))
    oq, os_ = orc.quant_weight(w)
    assert np.array_equal(host(gq), oq) and np.array_equal(host(gs), os_)
    gx = jet.quant_act(dev_bf16(x))
    ox = orc.quant_act(x)
    assert np.array_equal(host(gx["q_row"]), ox["q_row"]) and np.array_equal(host(gx["s_row"]), ox["s_row"])
    y = jet.fp8_linear_fwd(gx["q_row"], gx["s_row"], gq, gs)
    rows = ji.sample_rows(M, 12, 31 + M)
    ref = orc.gemm(ox["q_row"], ox["s_row"], oq, os_, rows=rows)
    check_gemm(host_bits(y)[rows], ref, f"8B {name} decode M={M}", operands=(ox["q_row"][rows], ox["s_row"][rows], oq, os_, False))


# ---- config 3: unified-flow invariance sweep ----

@pytest.mark.parametrize("idx", [0, 1, 4, 6])     # q, k, gate, down
def test_unified_flow_invariance_8b(jet, idx):
    """The same 128 token rows inside decode calls (M = 1, 8, 32, 128: skinny and strip
    kernels) and at seeded positions inside training-forward calls (M = 4096, 16384:
    persistent tile kernel) give identical output bytes; again after each of three
    synthetic weight updates with re-quantization."""
    name, N, K = ji.LAYER_8B[idx]
    R = ji.activations(128, K, ji.seed_for(3, idx, ji.TENSOR_X))
    w = ji.weights(N, K, ji.seed_for(3, idx, ji.TENSOR_W))
    qR = jet.quant_act(dev_bf16(R))
    gen = torch.Generator(device=DEV)
    for rnd in range(3):
        gq, gs = jet.quant_weight(dev_bf16(w))

        def fwd(qx, sx):
            return jet.fp8_linear_fwd(qx.contiguous(), sx.contiguous(), gq, gs)

        base = fwd(qR["q_row"], qR["s_row"]).view(torch.int16)            # M = 128
        for M in (1, 8, 32):
            perm = torch.from_numpy(np.random.default_rng(100 * rnd + M).permutation(128)[:M]).to(DEV)
            got = fwd(qR["q_row"][perm], qR["s_row"][perm]).view(torch.int16)
            assert torch.equal(got, base[perm]), f"{name} round {rnd}: decode M={M} differs from M=128"
        for M in (4096, 16384):
            # filler rows: seeded N(0,1) drawn on the GPU (only the GPU path consumes them)
            gen.manual_seed(ji.seed_for(3, idx, ji.TENSOR_POS) + M + rnd)
            other = torch.randn((M, K), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
            pos = torch.from_numpy(ji.row_positions(128, M, ji.seed_for(3, idx, ji.TENSOR_POS) + 7 * M + rnd)).to(DEV)
            other[pos] = dev_bf16(R)
            qo = jet.quant_act(other)
            assert torch.equal(qo["q_row"][pos], qR["q_row"]) and torch.equal(qo["s_row"][pos], qR["s_row"])
            got = fwd(qo["q_row"], qo["s_row"]).view(torch.int16)
            assert torch.equal(got[pos], base), f"{name} round {rnd}: training M={M} differs from decode"
            del other, qo, got
        w = ji.weight_update(w, ji.seed_for(3, idx, ji.TENSOR_UPDATE) + rnd)
