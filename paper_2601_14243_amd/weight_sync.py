"""Weight synchronisation between the trainer's bf16 master weights and the FP8 weights that
rollout and the training GEMMs read (Jet-RL Sec. 2.3: the updated actor's weights go to the
inference engine after every step; Sec. 4.1: the training graph differs from the rollout graph
only by the bf16 master copy; Sec. 4.2: the weights are quantized 128x128 during the parameter
update, which is compatible with tensor parallelism).

One layout serves every consumer: `q [N,K]` + `s [N/128,K/128]` is what jet_fp8_linear_fwd reads
in decode-shaped and training-shaped calls alike, and the transposed pair `qT [K,N]` +
`sT [K/128,N/128]` is what jet_fp8_linear_dgrad reads, so a synchronisation is nothing but one
jet_quant_weight per matrix into buffers that stay where they are -- no repacking, no second copy
for the rollout engine.  Under tensor parallelism a rank holds a 128-aligned shard of a master
weight (rows of a column-parallel matrix, columns of a row-parallel one); because the 128x128
blocks never straddle such a shard boundary, quantizing the shard gives exactly the shard of the
quantized whole, so every rank synchronises its own shard with the same call.
"""
from __future__ import annotations

import torch

from . import binding as jet

COLUMN_PARALLEL = ("q_proj", "k_proj", "v_proj", "gate_proj", "up_proj")   # split along N (output features)
ROW_PARALLEL = ("o_proj", "down_proj")                                      # split along K (input features)


def shard_shape(name: str, N: int, K: int, tp: int):
    """Shape of one rank's shard of matrix `name` under tensor parallelism of degree tp."""
    if tp == 1:
        return N, K
    n, k = (N // tp, K) if name in COLUMN_PARALLEL else (N, K // tp)
    if (N % tp if name in COLUMN_PARALLEL else K % tp) or n % 128 or k % 128:
        raise ValueError(f"{name} [{N},{K}] does not split into 128-aligned shards over {tp} ranks")
    return n, k


def shard_of(name: str, w: torch.Tensor, rank: int, tp: int) -> torch.Tensor:
    """The dense master shard of rank `rank` (what that rank's trainer holds)."""
    N, K = w.shape
    n, k = shard_shape(name, N, K, tp)
    if name in COLUMN_PARALLEL:
        return w[rank * n:(rank + 1) * n].contiguous()
    return w[:, rank * k:(rank + 1) * k].contiguous()


class WeightStore:
    """FP8 buffers of a whole model (or of one tensor-parallel rank's shards): per layer and matrix
    the tuple (q, s) or (q, s, qT, sT) that jet_quant_weight writes and the GEMM calls read."""

    def __init__(self, layer, n_layers: int, transposed: bool = True, tp: int = 1, device="cuda"):
        self.names = [name for name, _, _ in layer]
        self.transposed = transposed
        self.layers = []
        u8, f32 = torch.uint8, torch.float32
        for _ in range(n_layers):
            bufs = {}
            for name, N, K in layer:
                n, k = shard_shape(name, N, K, tp)
                t = [torch.empty((n, k), dtype=u8, device=device), torch.empty((n // 128, k // 128), dtype=f32, device=device)]
                if transposed:
                    t += [torch.empty((k, n), dtype=u8, device=device), torch.empty((k // 128, n // 128), dtype=f32, device=device)]
                bufs[name] = tuple(t)
            self.layers.append(bufs)

    def sync_layer(self, i: int, masters: dict) -> None:
        """masters: name -> bf16 master weight (this rank's dense shard) of layer i."""
        for name in self.names:
            jet.quant_weight(masters[name], transposed=self.transposed, out=self.layers[i][name])

    def sync(self, masters) -> None:
        """masters: one dict per layer.  Enqueues every re-quantization on the current stream."""
        for i, m in enumerate(masters):
            self.sync_layer(i, m)

    def bytes_moved(self) -> int:
        """HBM bytes of one synchronisation: bf16 masters read, codes and scales written."""
        total = 0
        for bufs in self.layers:
            for t in bufs.values():
                total += 2 * t[0].numel() + sum(x.numel() * x.element_size() for x in t)
        return total
