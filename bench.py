#!/usr/bin/env python3
"""Benchmark of the block-scaled FP8 linear layer on one MI355X.

One "step" is one pass of the whole hot path over the seven linears of an
8B-class decoder layer (hidden 4096, q/k/v/o, gate/up 14336, down) on synthetic
inputs already resident in HBM:
  training, M = 16384 tokens, per matrix: weight quantization with transposed copy,
  row quantization of X, FProp, fused row+column quantization of dY, DGrad,
  column re-quantization of the FP8-saved X, WGrad;
  rollout, M in {1, 8, 32, 128}: row quantization of the activations and FProp
  against the weights quantized above.
`value` is the GEMM work of the training part (3 GEMMs x 2 M N K per matrix)
divided by the time of the whole step (quantizers and decode calls included).

Prints ONE JSON line (see --help for the flags the driver passes).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5000.0     # MI355X dense FP8 MFMA peak
PEAK_HBM_GBPS = 8000.0
# HBM-side bytes per average FProp/DGrad launch of this workload come from two rocprofv3 --pmc runs
# of this script (FETCH_SIZE, WRITE_SIZE, each scaled by what it reads for a plain 1 GiB copy).  A
# profiler cannot run inside the timed region, so the figure is read from the committed summary of
# those runs (a line "TRAFFIC_BYTES_PER_FPROP_DGRAD_LAUNCH=<bytes> KERNELS_AT_COMMIT=<hash>"); it is
# null when the summary is missing.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "bench_8B_M16384_hbm_counters.txt")
DECODE_SUMMARY = os.path.join(ROOT, "profiles", "decode_8B_kernel_stats_and_fetch.txt")


def profiled_decode_traffic():
    """HBM reads of the largest decode launch (fused gate+up at M = 1), from the committed summary."""
    import re
    try:
        m = re.search(r"READ_BYTES_FUSED_GATE_UP_M1_LAUNCH=(\d+)\s+KERNELS_AT_COMMIT=(\w+)", open(DECODE_SUMMARY).read())
    except OSError:
        return None, None
    return (int(m.group(1)), m.group(2)) if m else (None, None)


def profiled_traffic():
    import re
    try:
        m = re.search(r"TRAFFIC_BYTES_PER_FPROP_DGRAD_LAUNCH=(\d+)\s+KERNELS_AT_COMMIT=(\w+)", open(TRAFFIC_SUMMARY).read())
    except OSError:
        return None, None
    return (int(m.group(1)), m.group(2)) if m else (None, None)

M_TRAIN = 16384
DECODE_M = (1, 8, 32, 128)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode-sweep", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the 32B-class GEMM pass and the weight re-quantization timing")
    ap.add_argument("--one", nargs=4, metavar=("KIND", "M", "N", "K"),
                    help="profiling mode: run ONE entry point a few times on synthetic data, then one plain "
                         "1 GiB device copy (its HBM counters calibrate FETCH_SIZE / WRITE_SIZE), and exit. "
                         "KIND: fwd, dgrad, wgrad, quant_row, quant_dual, quant_colT, quant_weight, rmsnorm_quant, "
                         "silu_mul_quant, silu_mul_bwd (for the last three M, N, K mean rows, -, columns)")
    ap.add_argument("--iters", type=int, default=5, help="launches in --one mode")
    ap.add_argument("--only-decode", action="store_true",
                    help="profiling mode: only the rollout (decode-shaped) sweep of the 8B-class layer")
    return ap.parse_args()


def run_one(torch, jet, kind, M, N, K, iters):
    """--one: a single entry point under the profiler (rocprofv3 -- python3 bench.py --one ...)."""
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
    elif kind == "silu_mul_bwd":
        gu = (torch.randn((M, 2 * K), generator=gen, device=dev) * 2.0).to(bf)
        dh = (torch.randn((M, K), generator=gen, device=dev) * 1e-3).to(bf)
        dgu = torch.empty_like(gu)
        fn = lambda: jet.silu_mul_bwd(gu[:, :K], gu[:, K:], dh, out=dgu)
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
    print(f"bench.py --one: {kind} M={M} N={N} K={K} x{iters}, then one 1 GiB device copy")


def make_inputs(torch, jet, M, layer):
    """Seeded synthetic tensors with the structure of jet_inputs' recipes, drawn on the
    GPU (same distributions; the parity tests use the host generator)."""
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    mats = []
    for idx, (name, N, K) in enumerate(layer):
        gen.manual_seed(2000 + 10 * idx)
        x = torch.randn((M, K), generator=gen, device=dev, dtype=torch.float32)
        n_out = -(-K // 100)
        cols = torch.randperm(K, generator=gen, device=dev)[:n_out]
        x[:, cols] *= 50.0
        x = x.to(torch.bfloat16)
        w = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
        dy = torch.randn((M, N), generator=gen, device=dev, dtype=torch.float32) * 1e-3
        mask = torch.rand((M, N), generator=gen, device=dev) < 0.005
        # Student-t(3) = normal / sqrt(chi2_3 / 3)
        z = torch.randn((M, N), generator=gen, device=dev)
        chi = (torch.randn((3, M, N), generator=gen, device=dev) ** 2).sum(0) / 3.0
        dy = torch.where(mask, 1e-3 * z / chi.sqrt(), dy).to(torch.bfloat16)
        del z, chi, mask
        u8, f32, bf = torch.uint8, torch.float32, torch.bfloat16
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        m = dict(name=name, N=N, K=K, x=x, w=w, dy=dy,
                 qx=dict(q_row=e((M, K), u8), s_row=e((M, K // 128), f32)),
                 qxT=dict(q_colT=e((K, M), u8), s_colT=e((K, M // 128), f32)),
                 qdy=dict(q_row=e((M, N), u8), s_row=e((M, N // 128), f32),
                          q_colT=e((N, M), u8), s_colT=e((N, M // 128), f32)),
                 qw=(e((N, K), u8), e((N // 128, K // 128), f32), e((K, N), u8), e((K // 128, N // 128), f32)),
                 y=e((M, N), bf), dx=e((M, K), bf), dw=e((N, K), bf), dec=[])
        for Md in DECODE_M:
            xd = x[:Md].contiguous()
            m["dec"].append(dict(M=Md, x=xd, q=dict(q_row=e((Md, K), u8), s_row=e((Md, K // 128), f32)),
                                 y=e((Md, N), bf)))
        mats.append(m)
    return mats


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU; run with --gpus 1 "
              "(no collective or multi-GPU path exists in this library)", file=sys.stderr)
        sys.exit(2)
    import torch
    import jet_inputs as ji
    import paper_2601_14243_amd as jet

    if not torch.cuda.is_available():
        print("bench.py: needs a GPU", file=sys.stderr)
        sys.exit(2)
    jet.lib()
    torch.cuda.set_device(0)
    if args.one:
        run_one(torch, jet, args.one[0], int(args.one[1]), int(args.one[2]), int(args.one[3]), args.iters)
        return
    layer = ji.LAYER_8B
    if args.only_decode:
        print(json.dumps({"decode": decode_sweep(torch, jet, layer)}))
        return
    M = M_TRAIN
    mats = make_inputs(torch, jet, M, layer)
    sum_nk = sum(N * K for _, N, K in layer)
    flops_step = 3 * 2 * M * sum_nk

    gemm_events = []   # (start, end, flops) around the block-scaled tile GEMM (FProp, DGrad)
    wgrad_events = []
    quant_events = []  # (start, end, bytes)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    per_matrix = {}    # (matrix, GEMM kind) -> [(start, end)]

    def timed(store, work, fn, tag=None):
        if store is None:
            fn()
            return
        a, b = ev(), ev()
        a.record()
        fn()
        b.record()
        store.append((a, b, work))
        if tag is not None:
            per_matrix.setdefault(tag, []).append((a, b))

    def step(record):
        ge = gemm_events if record else None
        we = wgrad_events if record else None
        qe = quant_events if record else None
        for m in mats:
            N, K = m["N"], m["K"]
            fl = 2 * M * N * K
            timed(qe, N * K * 4.0, lambda: jet.quant_weight(m["w"], transposed=True, out=m["qw"]))
            timed(qe, M * K * 3.03125, lambda: jet.quant_act(m["x"], out=m["qx"]))
            timed(ge, fl, lambda: jet.fp8_linear_fwd(m["qx"]["q_row"], m["qx"]["s_row"], m["qw"][0], m["qw"][1], out=m["y"]), (m["name"], "fwd"))
            timed(qe, M * N * 4.0625, lambda: jet.quant_act(m["dy"], row=True, col=True, out=m["qdy"]))
            timed(ge, fl, lambda: jet.fp8_linear_dgrad(m["qdy"]["q_row"], m["qdy"]["s_row"], m["qw"][2], m["qw"][3], out=m["dx"]), (m["name"], "dgrad"))
            timed(qe, M * K * 2.0625, lambda: jet.quant_act(m["qx"]["q_row"], m["qx"]["s_row"], row=False, col=True, out=m["qxT"]))
            timed(we, fl, lambda: jet.fp8_linear_wgrad(m["qdy"]["q_colT"], m["qdy"]["s_colT"], m["qxT"]["q_colT"], m["qxT"]["s_colT"], out=m["dw"]), (m["name"], "wgrad"))
            for d in m["dec"]:
                jet.quant_act(d["x"], out=d["q"])
                jet.fp8_linear_fwd(d["q"]["q_row"], d["q"]["s_row"], m["qw"][0], m["qw"][1], out=d["y"])

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    def rate(events):
        tot_t = sum(a.elapsed_time(b) for a, b, _ in events) * 1e-3
        tot_w = sum(w for _, _, w in events)
        return tot_w / tot_t, tot_t / len(events), tot_w / len(events)

    g_rate, g_avg_s, g_avg_fl = rate(gemm_events)
    # operands read once + bf16 output written once, per average FProp/DGrad launch
    tile_alg_bytes = sum((M * K + M * N) * (1 + 4 / 128) + 2 * (N * K + 4 * (N // 128) * (K // 128))
                         + 2 * M * N + 2 * M * K for _, N, K in layer) / (2 * len(layer))
    w_rate, w_avg_s, _ = rate(wgrad_events)
    q_rate, _, _ = rate(quant_events)
    gemm_time = sum(a.elapsed_time(b) for a, b, _ in gemm_events + wgrad_events) * 1e-3 / args.steps
    out = {
        "metric": "FP8 linear TFLOP/s (train fwd+bwd, M=16k) + decode GEMM HBM GB/s (M=1..128)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8_e4m3",
        "data": "synthetic",
        "config": {"workload": "8B-class decoder layer, 7 linears, training M=16384 (quantizers + "
                               "FProp + DGrad + WGrad) plus rollout FProp at M in {1,8,32,128}",
                   "sum_NK": sum_nk, "train_gemm_flop_per_step": flops_step},
        "train_gemm_only_tflops": round(flops_step / gemm_time / 1e12, 2),
        "fprop_dgrad_kernel_tflops": round(g_rate / 1e12, 2),
        "wgrad_kernel_tflops": round(w_rate / 1e12, 2),
        "quantizers_gbps": round(q_rate / 1e9, 1),
        "roofline": {"bound": "mfma", "kernel": "gemm_tile_kernel<block scales, 256x256> (FProp and DGrad launches)",
                     "achieved": round(g_rate / 1e12, 2), "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(g_rate / 1e12 / PEAK_FP8_TFLOPS, 4),
                     "avg_launch_ms": round(g_avg_s * 1e3, 4), "avg_launch_gflop": round(g_avg_fl / 1e9, 2),
                     "launches": len(gemm_events), "traffic": profiled_traffic()[0],
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, profiles/)",
                     "traffic_profiled_at_commit": profiled_traffic()[1],
                     "algorithmic_bytes": round(tile_alg_bytes)},
    }

    shape = {name: (N, K) for name, N, K in layer}
    out["per_matrix_tflops"] = {}
    for (name, kind), evs in per_matrix.items():
        t = sum(a.elapsed_time(b) for a, b in evs) * 1e-3 / len(evs)
        out["per_matrix_tflops"].setdefault(name, {})[kind] = round(2 * M * shape[name][0] * shape[name][1] / t / 1e12, 1)
    out["roofline"].update(sustained_mfma(torch, jet, g_rate))
    if not args.no_extras:
        out["requantize_8B_layer"] = requant_timing(torch, jet, mats)
    del mats
    torch.cuda.empty_cache()
    if not args.no_extras:
        out["fused_producers_8B_M16384"] = fused_producers(torch, jet, M)
        out["mlp_block_8B_M16384"] = mlp_block_timing(torch, jet, M)
        out["mismatch_probe"] = mismatch_probe(torch, jet)
        out["train_gemms_32B_M32768"] = train_gemms_32b(torch, jet)
        out["weight_sync"] = weight_sync_timing(torch, jet)
    if not args.no_decode_sweep:
        out["decode"] = decode_sweep(torch, jet, layer)
        out["decode_32B"] = decode_sweep_32b(torch, jet)
        out["decode_per_matrix_8B"] = decode_per_matrix(torch, jet, layer + FUSED_8B[:1] + FUSED_8B[2:3])
        d1 = out["decode"]["M=1"]
        out["roofline_decode"] = {"bound": "hbm", "kernel": "gemm_skinny_kernel (rollout FProp, M = 1, one 8B-class layer, "
                                  "weights streamed from HBM; q/k/v and gate/up each as one call)",
                                  "achieved": d1["fused_GB/s"], "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                  "frac": d1["fused_frac_hbm"], "seven_separate_calls_frac": d1["frac_hbm"],
                                  "traffic": None}
        rd, at = profiled_decode_traffic()
        if rd is not None:
            # per launch of the largest call of the layer (the per-layer figure above spans four launches)
            out["roofline_decode"]["traffic_fused_gate_up_launch"] = {
                "bytes_read": rd, "weight_bytes": 2 * 14336 * 4096, "profiled_at_commit": at,
                "source": "rocprofv3 FETCH_SIZE, profiles/decode_8B_kernel_stats_and_fetch.txt"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
        out["cpu_baseline"]["parity_config0"] = parity_config0(torch, jet)
    print(json.dumps(out))


def _time(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / reps


def requant_timing(torch, jet, mats):
    """Re-quantization of the seven weight matrices of the layer after an update (bf16 in, FP8
    codes + 128x128 scales out), without and with the transposed copy that DGrad reads."""
    nk = sum(m["N"] * m["K"] for m in mats)

    def plain():
        for m in mats:
            jet.quant_weight(m["w"], out=(m["qw"][0], m["qw"][1]))

    def both():
        for m in mats:
            jet.quant_weight(m["w"], transposed=True, out=m["qw"])

    t1, t2 = _time(torch, plain, 10), _time(torch, both, 10)
    return {"us_per_layer": round(t1 * 1e6, 1), "GB/s": round(nk * 3.0 / t1 / 1e9, 1),
            "with_transposed_copy_us_per_layer": round(t2 * 1e6, 1),
            "with_transposed_copy_GB/s": round(nk * 4.0 / t2 / 1e9, 1)}


def fused_producers(torch, jet, M):
    """The two operators in front of the layer's GEMMs writing FP8 directly (8B-class shapes):
    RMSNorm of the hidden states [M,4096] and SiLU(gate)*up of one [M,2*14336] projection output.
    GB/s = algorithmic bytes (bf16 in, codes + scales out) / time; the plain row quantizer on a
    stored bf16 tensor of the same shape is timed beside each."""
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(777)
    res = {}
    K = 4096
    # three tensors in turn (0.6 GB of traffic per round): no pass finds its input in the 256 MB memory-side cache
    xs = [torch.randn((M, K), generator=gen, device=dev).to(torch.bfloat16) for _ in range(3)]
    gamma = (1.0 + 0.1 * torch.randn((K,), generator=gen, device=dev)).to(torch.bfloat16)
    os_ = [jet.rmsnorm_quant(x, gamma, 1e-6) for x in xs]

    def fused():
        for x, o in zip(xs, os_):
            jet.rmsnorm_quant(x, gamma, 1e-6, out=o)

    def plain():
        for x, o in zip(xs, os_):
            jet.quant_act(x, out=o)

    t, tq = _time(torch, fused, 10) / 3, _time(torch, plain, 10) / 3
    by = M * K * (2 + 1 + 4 / 128)
    res["rmsnorm_quant"] = {"us": round(t * 1e6, 1), "GB/s": round(by / t / 1e9, 1),
                            "row_quantizer_alone_us": round(tq * 1e6, 1)}
    x, o = None, None
    del xs, os_
    del x, o
    K = 14336
    gu = (torch.randn((M, 2 * K), generator=gen, device=dev) * 2.0).to(torch.bfloat16)
    o = jet.silu_mul_quant(gu[:, :K], gu[:, K:])
    t = _time(torch, lambda: jet.silu_mul_quant(gu[:, :K], gu[:, K:], out=o), 10)
    h = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
    tq = _time(torch, lambda: jet.quant_act(h, out=o), 10)
    by = M * K * (4 + 1 + 4 / 128)
    res["silu_mul_quant"] = {"us": round(t * 1e6, 1), "GB/s": round(by / t / 1e9, 1),
                             "row_quantizer_alone_us": round(tq * 1e6, 1)}
    return res


def mlp_block_timing(torch, jet, M):
    """One MLP block of the 8B-class layer (hidden 4096, intermediate 14336) forward + backward with
    FP8-saved activations: every call of paper_2601_14243_amd.mlp_block (quantizers, three FProp-sized
    GEMMs forward, four backward, the element-wise backward), and the bytes saved between the passes."""
    from paper_2601_14243_amd import mlp_block
    dev, H, I = "cuda:0", 4096, 14336
    gen = torch.Generator(device=dev)
    gen.manual_seed(555)
    x = torch.randn((M, H), generator=gen, device=dev).to(torch.bfloat16)
    dy = (torch.randn((M, H), generator=gen, device=dev) * 1e-3).to(torch.bfloat16)
    W = mlp_block.MlpWeights((torch.randn((2 * I, H), generator=gen, device=dev) * 0.02).to(torch.bfloat16),
                             (torch.randn((H, I), generator=gen, device=dev) * 0.02).to(torch.bfloat16))
    state = {}

    def fwd():
        state["y"], state["saved"] = mlp_block.forward(x, W)

    def bwd():
        state["out"] = mlp_block.backward(state["saved"], dy, W)

    t_f = _time(torch, fwd, 5)
    t_b = _time(torch, bwd, 5)
    fl_f, fl_b = 2.0 * M * 3 * I * H, 2 * 2.0 * M * 3 * I * H
    sb = mlp_block.saved_bytes(M, H, I)
    state.clear()
    torch.cuda.empty_cache()
    return {"forward_ms": round(t_f * 1e3, 3), "backward_ms": round(t_b * 1e3, 3),
            "forward_tflops": round(fl_f / t_f / 1e12, 1), "backward_tflops": round(fl_b / t_b / 1e12, 1),
            "block_tflops": round((fl_f + fl_b) / (t_f + t_b) / 1e12, 1),
            "saved_activation_MB": round(sb["fp8_saved"] / 1e6, 1), "saved_if_bf16_MB": round(sb["bf16_saved"] / 1e6, 1),
            "saved_ratio": round(sb["ratio"], 3)}


def weight_sync_timing(torch, jet):
    """Whole-model re-quantization at the parameter update (paper_2601_14243_amd.weight_sync): every
    linear of every layer from its bf16 master into the FP8 buffers rollout and training read, with
    and without the transposed copies DGrad needs.  8B-class: 32 layers; 32B-class: 64 layers."""
    import jet_inputs as ji
    from paper_2601_14243_amd import weight_sync as ws
    dev = "cuda:0"
    res = {}
    for tag, layer, n_layers in (("8B_32_layers", ji.LAYER_8B, 32), ("32B_64_layers", ji.LAYER_32B, 64)):
        gen = torch.Generator(device=dev)
        gen.manual_seed(4321)
        # one set of masters per layer shape, reused by every layer (the kernels read 2 bytes per weight
        # either way; distinct FP8 buffers per layer keep the written footprint that of the whole model)
        masters = {name: (torch.randn((N, K), generator=gen, device=dev) * 0.02).to(torch.bfloat16) for name, N, K in layer}
        r = {}
        for transposed in (False, True):
            store = ws.WeightStore(layer, n_layers, transposed=transposed)
            t = _time(torch, lambda: store.sync([masters] * n_layers), 3)
            key = "with_transposed_copy" if transposed else "forward_layout_only"
            r[key] = {"ms": round(t * 1e3, 2), "GB/s": round(store.bytes_moved() / t / 1e9, 1),
                      "GB_moved": round(store.bytes_moved() / 1e9, 2)}
            del store
            torch.cuda.empty_cache()
        res[tag] = r
        del masters
        torch.cuda.empty_cache()
    return res


def mismatch_probe(torch, jet):
    """The property the unified flow exists for, on a synthetic stack of 8 MLP blocks (hidden 4096,
    intermediate 14336; RMSNorm -> FP8, gate/up FProp, SiLU*up -> FP8, down FProp, residual add):
    64 token rows pushed through as a decode-shaped batch and at seeded positions inside a
    training-shaped batch of 4096 rows.  Reported per depth: the largest byte-level difference
    between the two (must be zero), and, for scale, the relative distance of the FP8 stream from the
    same stack evaluated with bf16 GEMMs (torch.matmul) -- the rollout/training gap a mixed
    BF16-train / FP8-rollout setup would carry."""
    dev, H, I, L, T, MB = "cuda:0", 4096, 14336, 8, 64, 4096
    gen = torch.Generator(device=dev)
    gen.manual_seed(31337)
    blocks = []
    for _ in range(L):
        gamma = (1.0 + 0.1 * torch.randn((H,), generator=gen, device=dev)).to(torch.bfloat16)
        w_gu = (torch.randn((2 * I, H), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
        w_d = (torch.randn((H, I), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
        blocks.append((gamma, w_gu, w_d, jet.quant_weight(w_gu), jet.quant_weight(w_d)))

    def fp8_stack(x):
        outs = []
        for gamma, _, _, (qgu, sgu), (qd, sd) in blocks:
            h = jet.rmsnorm_quant(x, gamma, 1e-6)
            gu = jet.fp8_linear_fwd(h["q_row"], h["s_row"], qgu, sgu)
            a = jet.silu_mul_quant(gu[:, :I], gu[:, I:])
            x = x + jet.fp8_linear_fwd(a["q_row"], a["s_row"], qd, sd)
            outs.append(x)
        return outs

    def bf16_stack(x):
        outs = []
        for gamma, w_gu, w_d, _, _ in blocks:
            xf = x.float()
            n = (xf * torch.rsqrt(xf.pow(2).mean(-1, keepdim=True) + 1e-6)).to(torch.bfloat16) * gamma
            gu = n @ w_gu.t()
            a = torch.nn.functional.silu(gu[:, :I]) * gu[:, I:]
            x = x + a @ w_d.t()
            outs.append(x)
        return outs

    tokens = torch.randn((T, H), generator=gen, device=dev).to(torch.bfloat16)
    batch = torch.randn((MB, H), generator=gen, device=dev).to(torch.bfloat16)
    pos = torch.randperm(MB, generator=gen, device=dev)[:T]
    batch[pos] = tokens
    dec, trn, ref = fp8_stack(tokens), fp8_stack(batch), bf16_stack(tokens)
    same = [int((d.view(torch.int16) != t[pos].view(torch.int16)).sum().item()) for d, t in zip(dec, trn)]
    rel = [round(float(((d.float() - r.float()).norm() / r.float().norm()).item()), 5) for d, r in zip(dec, ref)]
    return {"blocks": L, "tokens": T, "training_batch_rows": MB,
            "differing_bf16_values_decode_vs_training_by_depth": same,
            "fp8_vs_bf16_gemm_relative_l2_by_depth": rel}


def train_gemms_32b(torch, jet):
    """FProp, DGrad and WGrad of the seven 32B-class matrices at M = 32768 (long rollouts packed
    into one training batch), GEMM kernels only, one matrix resident at a time."""
    import jet_inputs as ji
    dev, M = "cuda:0", 32768
    gen = torch.Generator(device=dev)
    t_tot, fl_tot, per = 0.0, 0.0, {}
    for idx, (name, N, K) in enumerate(ji.LAYER_32B):
        gen.manual_seed(4000 + idx)
        x = torch.randn((M, K), generator=gen, device=dev).to(torch.bfloat16)
        w = (torch.randn((N, K), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
        dy = (torch.randn((M, N), generator=gen, device=dev) * 1e-3).to(torch.bfloat16)
        qx = jet.quant_act(x)
        qxT = jet.quant_act(qx["q_row"], qx["s_row"], row=False, col=True)
        qdy = jet.quant_act(dy, row=True, col=True)
        qw = jet.quant_weight(w, transposed=True)
        del x, w, dy
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
        t = (_time(torch, lambda: jet.fp8_linear_fwd(qx["q_row"], qx["s_row"], qw[0], qw[1], out=y), 3)
             + _time(torch, lambda: jet.fp8_linear_dgrad(qdy["q_row"], qdy["s_row"], qw[2], qw[3], out=dx), 3)
             + _time(torch, lambda: jet.fp8_linear_wgrad(qdy["q_colT"], qdy["s_colT"], qxT["q_colT"], qxT["s_colT"], out=dw), 3))
        fl = 3 * 2.0 * M * N * K
        per[name] = round(fl / t / 1e12, 1)
        t_tot += t
        fl_tot += fl
        del qx, qxT, qdy, qw, y, dx, dw
        torch.cuda.empty_cache()
    return {"tflops": round(fl_tot / t_tot / 1e12, 1), "ms_per_layer": round(t_tot * 1e3, 2),
            "frac_of_peak": round(fl_tot / t_tot / 1e12 / PEAK_FP8_TFLOPS, 4), "per_matrix_tflops": per}


def sustained_mfma(torch, jet, achieved_flops):
    """Context for `frac`: the rate the same FP8 matrix-core instruction sustains on this machine
    from registers alone (no LDS, no memory), with pseudo-random and with all-zero operands,
    and the shader clock the driver reports meanwhile (null if it is not readable).  Operand values change the power the
    matrix cores draw and with it the clock; the published peak is at the full 2.4 GHz."""
    import glob
    import re
    import threading

    from paper_2601_14243_amd import probe

    def sclk():
        # current shader clock from sysfs (the level marked '*'); no child process is started
        best = None
        for f in glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"):
            try:
                for line in open(f).read().splitlines():
                    m = re.match(r"\s*\S+:\s*(\d+)\s*[Mm][Hh]z\s*\*", line)
                    if m:
                        best = max(best or 0, int(m.group(1)))
            except OSError:
                pass
        return best

    res = {}
    for name, zero in (("random", False), ("zero", True)):
        clk = []
        th = threading.Thread(target=lambda: (time.sleep(0.25), clk.append(sclk())))
        probe.probe_mfma_rate(workgroups=1024, iters=4000, zero_data=zero, repeats=3)    # bring the clock to its steady state
        th.start()
        r = probe.probe_mfma_rate(workgroups=1024, iters=4000, zero_data=zero, repeats=40)
        th.join()
        res[f"mfma_only_{name}_operands_tflops"] = round(r / 1e12, 1)
        res[f"mfma_only_{name}_operands_sclk_mhz"] = clk[0] if clk else None
    res["frac_of_mfma_only_random_operands"] = round(achieved_flops / 1e12 / res["mfma_only_random_operands_tflops"], 4)
    return res


FUSED_8B = (("qkv_proj", 6144, 4096), ("o_proj", 4096, 4096), ("gate_up_proj", 28672, 4096),
            ("down_proj", 4096, 14336))


def decode_sweep(torch, jet, layer, rotations=4):
    """Rollout FProp over the layer with `rotations` distinct weight sets (> 256 MB each
    pass, so weights come from HBM, not from the last-level cache); one HIP graph per M
    replayed several times; GB/s = algorithmic bytes / time.  Reported for the seven
    separate linears and for the same layer with q/k/v and gate/up concatenated along N
    (they share their input), which is how a serving engine calls them."""
    res = _decode_sweep(torch, jet, layer, rotations)
    fused = _decode_sweep(torch, jet, FUSED_8B, rotations)
    for k, v in fused.items():
        res[k]["fused_us_per_layer"] = v["us_per_layer"]
        res[k]["fused_GB/s"] = v["GB/s"]
        res[k]["fused_frac_hbm"] = v["frac_hbm"]
    return res


def decode_per_matrix(torch, jet, layer, ms=(1, 32, 128)):
    """Each matrix of the layer by itself, decode-shaped, against so many distinct copies of it (> 600 MB)
    that every weight byte comes from HBM; one HIP graph per (matrix, M).  us per call and GB/s."""
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(777)
    res = {}
    for name, N, K in layer:
        copies = max(3, int(600e6 // (N * K)) + 1)
        ws = [jet.quant_weight((torch.randn((N, K), generator=gen, device=dev) * 0.02).to(torch.bfloat16))
              for _ in range(copies)]
        res[name] = {}
        for Md in ms:
            a = jet.quant_act(torch.randn((Md, K), generator=gen, device=dev).to(torch.bfloat16))
            y = torch.empty((Md, N), dtype=torch.bfloat16, device=dev)

            def run():
                for q, sc in ws:
                    jet.fp8_linear_fwd(a["q_row"], a["s_row"], q, sc, out=y)

            st = torch.cuda.Stream()
            st.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(st):
                run()
            torch.cuda.current_stream().wait_stream(st)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run()
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / (10 * copies)
            by = N * K + 4 * (N // 128) * (K // 128) + Md * K + 4 * Md * (K // 128) + 2 * Md * N
            res[name][f"M={Md}"] = {"us": round(t * 1e6, 2), "GB/s": round(by / t / 1e9)}
        del ws
        torch.cuda.empty_cache()
    return res


def decode_sweep_32b(torch, jet):
    """The same sweep on the 32B-class layer (hidden 5120, intermediate 27648) at M in {1, 64, 256};
    one layer is 488 MB of weights, so two rotating sets keep every pass out of the caches."""
    import jet_inputs as ji
    return _decode_sweep(torch, jet, ji.LAYER_32B, 2, ms=(1, 64, 256))


def _decode_sweep(torch, jet, layer, rotations, ms=None):
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    sets = []
    for _ in range(rotations):
        ws = []
        for _, N, K in layer:
            w = (torch.randn((N, K), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
            ws.append(jet.quant_weight(w))
            del w
        sets.append(ws)
    res = {}
    for Md in (ms or DECODE_M + (16,)):
        xs, acts, outs = [], [], []
        for _, N, K in layer:
            x = torch.randn((Md, K), generator=gen, device=dev).to(torch.bfloat16)
            xs.append(x)
            acts.append(jet.quant_act(x))
            outs.append(torch.empty((Md, N), dtype=torch.bfloat16, device=dev))

        def gemms():
            for ws in sets:
                for (q, s), a, y in zip(ws, acts, outs):
                    jet.fp8_linear_fwd(a["q_row"], a["s_row"], q, s, out=y)

        def quant_and_gemms():                      # a1 + a4: the row quantizer in front of every GEMM
            for ws in sets:
                for (q, s), x, a, y in zip(ws, xs, acts, outs):
                    jet.quant_act(x, out=a)
                    jet.fp8_linear_fwd(a["q_row"], a["s_row"], q, s, out=y)

        def graph_time(run):
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                run()
            torch.cuda.current_stream().wait_stream(s)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run()
            g.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 10
            a.record()
            for _ in range(reps):
                g.replay()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e-3 / (reps * rotations)

        t_layer, t_q = graph_time(gemms), graph_time(quant_and_gemms)
        by = sum(N * K + 4 * (N // 128) * (K // 128) + Md * K + 4 * Md * (K // 128) + 2 * Md * N for _, N, K in layer)
        res[f"M={Md}"] = {"us_per_layer": round(t_layer * 1e6, 2), "GB/s": round(by / t_layer / 1e9, 1),
                          "frac_hbm": round(by / t_layer / 1e9 / PEAK_HBM_GBPS, 4),
                          "with_row_quantizer_us_per_layer": round(t_q * 1e6, 2)}
    return res


def cpu_baseline():
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the small
    configuration's shapes (N = K = 1024) with M scaled to roughly 15 s of CPU work."""
    import jet_inputs as ji
    import oracle as orc

    def run(M, N, K):
        x, w, dy = ji.activations(M, K, 1), ji.weights(N, K, 2), ji.grads(M, N, 3)
        t0 = time.perf_counter()
        qx = orc.quant_act(x)
        qw, sw, qwT, swT = orc.quant_weight(w, transposed=True)
        qdy = orc.quant_act(dy, row=True, col=True)
        qxT = orc.quant_act(qx["q_row"], qx["s_row"], src=orc.SRC_FP8_ROW, row=False, col=True)
        orc.fp8_linear_fwd(qx["q_row"], qx["s_row"], qw, sw)
        orc.fp8_linear_dgrad(qdy["q_row"], qdy["s_row"], qwT, swT)
        orc.fp8_linear_wgrad(qdy["q_colT"], qdy["s_colT"], qxT["q_colT"], qxT["s_colT"])
        return time.perf_counter() - t0

    N = K = 1024
    all_threads = orc.num_threads()
    # two small runs separate the fixed part (weight quantization) from the cost per 128 rows
    t1, t3 = run(128, N, K), run(384, N, K)
    per = max((t3 - t1) / 2.0, 1e-3)
    k = int(min(400, max(1, round((12.0 - max(t1 - per, 0.0)) / per))))
    M = 128 * k
    t = run(M, N, K)
    fl = 3 * 2 * M * N * K
    res = {"value": round(fl / t / 1e12, 6), "unit": "TFLOP/s", "cores": all_threads, "kind": "oracle",
           "sample": f"one linear N=K=1024, M={M}: quantizers + FProp + DGrad + WGrad, {t:.1f} s"}
    # the same oracle on one thread, on a sample sized for a few seconds
    orc.set_num_threads(1)
    M1 = 128 * max(1, int(round(M / all_threads / 128 / 3)))
    t = run(M1, N, K)
    orc.set_num_threads(all_threads)
    res["one_thread"] = {"value": round(3 * 2 * M1 * N * K / t / 1e12, 6), "unit": "TFLOP/s", "cores": 1,
                         "sample": f"the same linear at M={M1}, {t:.1f} s"}
    return res


def parity_config0(torch, jet):
    """Part of the CPU-baseline leg (the only place this script touches the oracle): the small
    configuration (M=256, N=K=1024) on the GPU against the oracle -- FP8 bytes and scales equal,
    share of outputs within 2 bf16 ulp of the oracle's binary32 reference order, worst element."""
    import numpy as np
    import jet_inputs as ji
    import oracle as orc
    M, N, K = 256, 1024, 1024
    x, w = ji.activations(M, K, ji.seed_for(0, 0, ji.TENSOR_X)), ji.weights(N, K, ji.seed_for(0, 0, ji.TENSOR_W))
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to("cuda:0")
    gx, (gq, gs) = jet.quant_act(to_dev(x)), jet.quant_weight(to_dev(w))
    y = jet.fp8_linear_fwd(gx["q_row"], gx["s_row"], gq, gs).view(torch.int16).cpu().numpy().view(np.uint16)
    ox = orc.quant_act(x)
    oq, os_ = orc.quant_weight(w)
    ref = orc.gemm(ox["q_row"], ox["s_row"], oq, os_)
    yf = (y.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    acc = ref["acc"].astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(acc), 2.0 ** -126))) - 7)
    err = np.abs(yf - acc) / ulp
    return {"fp8_bytes_and_scales_equal": bool(np.array_equal(gx["q_row"].cpu().numpy(), ox["q_row"])
                                               and np.array_equal(gx["s_row"].cpu().numpy(), ox["s_row"])
                                               and np.array_equal(gq.cpu().numpy(), oq) and np.array_equal(gs.cpu().numpy(), os_)),
            "gemm_within_2_bf16_ulp_frac": round(float((err <= 2.0).mean()), 6),
            "gemm_bf16_equal_frac": round(float((y == ref["out"]).mean()), 6),
            "gemm_worst_ulps": round(float(err.max()), 1),
            "note": "misses are cancellation cases (tiny outputs); tests hold every element to the modelled matrix-core instruction bit for bit"}


if __name__ == "__main__":
    main()
