"""The entry points under HIP graph capture and on a stream of the caller's: the library neither
allocates nor synchronises (include/jet.h), so a captured sequence of calls must replay to the
same bytes as the eager calls, replay after replay, with the program's own eager work and
synchronisations in between."""
import pytest
import torch

import jet_inputs as ji
from jet_testlib import dev_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jet():
    import paper_2601_14243_amd as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def _bits(t):
    return t.contiguous().view(torch.int16)


def test_mlp_block_forward_and_backward_replayed_from_a_graph(jet):
    from paper_2601_14243_amd import mlp_block
    M, H, I = 256, 512, 1024
    w = mlp_block.MlpWeights(dev_bf16(ji.weights(2 * I, H, 11)), dev_bf16(ji.weights(H, I, 12)))
    inputs = [(dev_bf16(ji.activations(M, H, 20 + i)), dev_bf16(ji.grads(M, H, 30 + i))) for i in range(3)]
    x, dy = inputs[0][0].clone(), inputs[0][1].clone()

    def run():
        y, saved = mlp_block.forward(x, w)
        g = mlp_block.backward(saved, dy, w)
        return y, g["dx"], g["dw_gu"], g["dw_d"]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up on the capture stream
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        outs = run()
    for rep in range(6):
        xi, dyi = inputs[rep % 3]
        x.copy_(xi)
        dy.copy_(dyi)
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        want = run()                                    # the program's own eager work between the replays
        torch.cuda.synchronize()
        for name, a, b in zip(("y", "dx", "dw_gu", "dw_d"), got, want):
            assert torch.equal(_bits(a), _bits(b)), f"replay {rep}: {name} differs from the eager call"


def test_decode_calls_on_a_side_stream_and_in_a_graph(jet):
    N, K = 1024, 2048
    qw, sw = jet.quant_weight(dev_bf16(ji.weights(N, K, 41)))
    xs = [dev_bf16(ji.activations(Md, K, 50 + Md)) for Md in (1, 5, 27, 100)]
    eager = []
    for xd in xs:
        a = jet.quant_act(xd)
        eager.append(jet.fp8_linear_fwd(a["q_row"], a["s_row"], qw, sw))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        on_side = []
        for xd in xs:
            a = jet.quant_act(xd)
            on_side.append(jet.fp8_linear_fwd(a["q_row"], a["s_row"], qw, sw))
    side.synchronize()
    for e, s in zip(eager, on_side):
        assert torch.equal(_bits(e), _bits(s))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = []
        for xd in xs:
            a = jet.quant_act(xd)
            captured.append(jet.fp8_linear_fwd(a["q_row"], a["s_row"], qw, sw))
    for rep in range(3):
        for c in captured:
            c.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for e, c in zip(eager, captured):
            assert torch.equal(_bits(e), _bits(c)), f"replay {rep}"
