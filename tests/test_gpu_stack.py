"""The unified precision flow through a stack of MLP blocks (Sec. 4.1: the rollout graph is a
subgraph of the training forward graph, so a token must get the same numbers in both): the same
token rows pushed through L blocks of  RMSNorm -> FP8 | gate/up FProp | SiLU*up -> FP8 | down
FProp | residual add  as decode-shaped batches (M = 1 ... 100: skinny and strip kernels) and
inside training-shaped batches (M = 640, 4096: tile kernels) must agree in every byte at every
depth.  Any shape-dependent arithmetic anywhere in the chain would be amplified by the
re-quantizations of the following blocks, which is the mismatch the method removes."""
import numpy as np
import pytest
import torch

import jet_inputs as ji
from jet_testlib import DEV, dev_bf16

pytestmark = pytest.mark.gpu

HIDDEN, INTER, BLOCKS, TOKENS = 1024, 3584, 6, 100


@pytest.fixture(scope="module")
def jet():
    import paper_2601_14243_amd as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def _weights(jet):
    blocks = []
    for b in range(BLOCKS):
        gamma = dev_bf16(ji.norm_weight(HIDDEN, seed=9000 + b).reshape(1, HIDDEN)).reshape(HIDDEN)
        w_gu = jet.quant_weight(dev_bf16(ji.weights(2 * INTER, HIDDEN, seed=9100 + b)))
        w_d = jet.quant_weight(dev_bf16(ji.weights(HIDDEN, INTER, seed=9200 + b)))
        blocks.append((gamma, w_gu, w_d))
    return blocks


def _forward(jet, blocks, x):
    """Returns the residual stream after every block (bf16 [M, HIDDEN] each)."""
    out = []
    for gamma, (q_gu, s_gu), (q_d, s_d) in blocks:
        h = jet.rmsnorm_quant(x, gamma, 1e-6)
        gu = jet.fp8_linear_fwd(h["q_row"], h["s_row"], q_gu, s_gu)            # [M, 2 INTER], gate | up
        a = jet.silu_mul_quant(gu[:, :INTER], gu[:, INTER:])
        d = jet.fp8_linear_fwd(a["q_row"], a["s_row"], q_d, s_d)
        x = x + d                                                               # element-wise bf16 add
        out.append(x)
    return out


def test_decode_and_training_shapes_agree_through_a_stack_of_blocks(jet):
    blocks = _weights(jet)
    tokens = dev_bf16(ji.activations(TOKENS, HIDDEN, seed=9300))
    base = _forward(jet, blocks, tokens)                                        # M = 100: strip kernel
    assert all(torch.isfinite(t.float()).all() for t in base)
    # the blocks do something: the stream moves away from its input
    assert (base[-1].float() - tokens.float()).abs().mean() > 0.05

    for M in (1, 8, 32, 77):                                                    # decode-shaped subsets
        pick = torch.from_numpy(np.random.default_rng(M).permutation(TOKENS)[:M]).to(DEV)
        got = _forward(jet, blocks, tokens[pick].contiguous())
        for depth, (g, b) in enumerate(zip(got, base)):
            assert torch.equal(g.view(torch.int16), b[pick].view(torch.int16)), f"M={M}: differs after block {depth}"

    gen = torch.Generator(device=DEV)
    for M in (640, 4096):                                                       # training-shaped batches
        gen.manual_seed(9400 + M)
        batch = torch.randn((M, HIDDEN), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
        pos = torch.from_numpy(ji.row_positions(TOKENS, M, seed=9500 + M)).to(DEV)
        batch[pos] = tokens
        got = _forward(jet, blocks, batch)
        for depth, (g, b) in enumerate(zip(got, base)):
            assert torch.equal(g[pos].view(torch.int16), b.view(torch.int16)), f"M={M}: differs after block {depth}"
