"""The library under HIP graph capture: every entry point only enqueues kernels on the caller's
stream (no allocation, no synchronisation, no memset), so a captured sequence must replay to the
bytes of the eager run, on every replay, also with other work and synchronisations in between."""
import pytest
import torch

import jet_inputs as ji
from jet_testlib import DEV, dev_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jet():
    import paper_2601_14243_amd as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def test_a_captured_layer_step_replays_to_the_eager_bytes(jet):
    M, N, K = 384, 512, 1024
    x = dev_bf16(ji.activations(M, K, seed=61))
    w = dev_bf16(ji.weights(N, K, seed=62))
    dy = dev_bf16(ji.grads(M, N, seed=63))
    gamma = dev_bf16(ji.norm_weight(K, seed=64).reshape(1, K)).reshape(K)
    gu = dev_bf16(ji.mlp_intermediate(M, K, seed=65))

    bufs = {
        "qx": jet.quant_act(x), "qw": jet.quant_weight(w, transposed=True),
        "qdy": jet.quant_act(dy, row=True, col=True),
        "y": torch.empty((M, N), dtype=torch.bfloat16, device=DEV),
        "y1": torch.empty((1, N), dtype=torch.bfloat16, device=DEV),
        "y40": torch.empty((40, N), dtype=torch.bfloat16, device=DEV),
        "dx": torch.empty((M, K), dtype=torch.bfloat16, device=DEV),
        "dw": torch.empty((N, K), dtype=torch.bfloat16, device=DEV),
    }
    bufs["qxT"] = jet.quant_act(bufs["qx"]["q_row"], bufs["qx"]["s_row"], row=False, col=True)
    bufs["rn"] = jet.rmsnorm_quant(x, gamma, 1e-6)
    bufs["sm"] = jet.silu_mul_quant(gu[:, :K], gu[:, K:])

    def step():
        b = bufs
        jet.quant_act(x, out=b["qx"])
        jet.quant_weight(w, transposed=True, out=b["qw"])
        jet.quant_act(dy, row=True, col=True, out=b["qdy"])
        jet.quant_act(b["qx"]["q_row"], b["qx"]["s_row"], row=False, col=True, out=b["qxT"])
        jet.rmsnorm_quant(x, gamma, 1e-6, out=b["rn"])
        jet.silu_mul_quant(gu[:, :K], gu[:, K:], out=b["sm"])
        jet.fp8_linear_fwd(b["qx"]["q_row"], b["qx"]["s_row"], b["qw"][0], b["qw"][1], out=b["y"])      # tile kernel
        jet.fp8_linear_fwd(b["qx"]["q_row"][:1], b["qx"]["s_row"][:1], b["qw"][0], b["qw"][1], out=b["y1"])   # skinny
        jet.fp8_linear_fwd(b["qx"]["q_row"][:40], b["qx"]["s_row"][:40], b["qw"][0], b["qw"][1], out=b["y40"])  # strip
        jet.fp8_linear_dgrad(b["qdy"]["q_row"], b["qdy"]["s_row"], b["qw"][2], b["qw"][3], out=b["dx"])
        jet.fp8_linear_wgrad(b["qdy"]["q_colT"], b["qdy"]["s_colT"], b["qxT"]["q_colT"], b["qxT"]["s_colT"], out=b["dw"])

    def tensors():
        b = bufs
        return [b["qx"]["q_row"], b["qx"]["s_row"], *b["qw"], b["qdy"]["q_row"], b["qdy"]["s_row"],
                b["qdy"]["q_colT"], b["qdy"]["s_colT"], b["qxT"]["q_colT"], b["qxT"]["s_colT"],
                b["rn"]["q_row"], b["rn"]["s_row"], b["sm"]["q_row"], b["sm"]["s_row"],
                b["y"], b["y1"], b["y40"], b["dx"], b["dw"]]

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone().view(torch.uint8) for t in tensors()]

    def scrub():
        for t in tensors():
            t.view(torch.uint8).fill_(0xA5)

    step()
    eager = snapshot()

    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()

    for replay in range(4):
        scrub()
        if replay % 2:                       # eager work of the program between replays
            torch.cuda.synchronize()
            _ = (x.float() * 2).sum().item()
        g.replay()
        got = snapshot()
        for i, (a, b) in enumerate(zip(got, eager)):
            assert torch.equal(a, b), f"replay {replay}: tensor {i} differs from the eager run"
