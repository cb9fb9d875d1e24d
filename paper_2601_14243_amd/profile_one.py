"""Run one entry point of libjet a few times on synthetic data, for rocprofv3.

    python3 paper_2601_14243_amd/profile_one.py fwd 16384 4096 4096 [iters]
    kinds: fwd, dgrad, wgrad, quant_row, quant_dual, quant_colT, quant_weight, rmsnorm_quant,
    silu_mul_quant (for these two M, N, K mean rows, -, columns)

Also launches one plain device-to-device copy of 1 GiB (torch's copy kernel): the
HBM counters (FETCH_SIZE, WRITE_SIZE) of that launch, divided by its known size,
give the scale factor for the counters of the profiled kernel.
"""
from __future__ import annotations

import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import paper_2601_14243_amd as jet  # noqa: E402


def main(argv):
    kind = argv[1]
    M, N, K = int(argv[2]), int(argv[3]), int(argv[4])
    iters = int(argv[5]) if len(argv) > 5 else 5
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    bf = torch.bfloat16
    x = torch.randn((M, K), generator=gen, device=dev).to(bf)
    w = (torch.randn((N, K), generator=gen, device=dev) * 0.02).to(bf)
    dy = (torch.randn((M, N), generator=gen, device=dev) * 1e-3).to(bf)
    qx = jet.quant_act(x)
    qw = jet.quant_weight(w, transposed=True)
    if kind == "fwd":
        y = torch.empty((M, N), device=dev, dtype=bf)
        fn = lambda: jet.fp8_linear_fwd(qx["q_row"], qx["s_row"], qw[0], qw[1], out=y)
    elif kind == "dgrad":
        qdy = jet.quant_act(dy)
        dx = torch.empty((M, K), device=dev, dtype=bf)
        fn = lambda: jet.fp8_linear_dgrad(qdy["q_row"], qdy["s_row"], qw[2], qw[3], out=dx)
    elif kind == "wgrad":
        qdy = jet.quant_act(dy, row=False, col=True)
        qxT = jet.quant_act(qx["q_row"], qx["s_row"], row=False, col=True)
        dw = torch.empty((N, K), device=dev, dtype=bf)
        fn = lambda: jet.fp8_linear_wgrad(qdy["q_colT"], qdy["s_colT"], qxT["q_colT"], qxT["s_colT"], out=dw)
    elif kind == "quant_row":
        fn = lambda: jet.quant_act(x, out=qx)
    elif kind == "quant_dual":
        qdy = jet.quant_act(dy, row=True, col=True)
        fn = lambda: jet.quant_act(dy, row=True, col=True, out=qdy)
    elif kind == "quant_colT":
        qxT = jet.quant_act(qx["q_row"], qx["s_row"], row=False, col=True)
        fn = lambda: jet.quant_act(qx["q_row"], qx["s_row"], row=False, col=True, out=qxT)
    elif kind == "quant_weight":
        fn = lambda: jet.quant_weight(w, transposed=True, out=qw)
    elif kind == "rmsnorm_quant":
        gamma = (1.0 + 0.1 * torch.randn((K,), generator=gen, device=dev)).to(bf)
        fn = lambda: jet.rmsnorm_quant(x, gamma, 1e-6, out=qx)
    elif kind == "silu_mul_quant":
        gu = (torch.randn((M, 2 * K), generator=gen, device=dev) * 2.0).to(bf)
        fn = lambda: jet.silu_mul_quant(gu[:, :K], gu[:, K:], out=qx)
    else:
        raise SystemExit(f"unknown kind {kind}")
    torch.cuda.synchronize()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    # calibration copy: 1 GiB read + 1 GiB written
    a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    a.fill_(1)
    torch.cuda.synchronize()
    b.copy_(a)
    torch.cuda.synchronize()
    print(f"profile_one: {kind} M={M} N={N} K={K} x{iters}, then one 1 GiB device copy")


if __name__ == "__main__":
    main(sys.argv)
