"""Composition of the library's entry points into the MLP block of a decoder layer with
FP8-saved activations (Jet-RL Sec. 4.1: the tensors saved for the backward GEMMs are the FP8 ones
the forward GEMMs consumed; gradients between operators stay bf16; Sec. 4.2: one fused row +
column quantization per gradient, column re-quantization of the saved FP8 activations).

Every arithmetic step is one call into libjet.so; this module only orders the calls and keeps
the saved tensors.  Layout: the gate and up projections are one weight [2 I, H] (gate rows first),
so their output is one [M, 2 I] tensor and their backward is one DGrad and one WGrad.

    forward :  x --row quant--> (qx)  --FProp W_gu-->  gu  --SiLU*mul, row quant--> (qh)  --FProp W_d-->  y
    saved   :  qx (FP8 + scales), gu (bf16, input of the element-wise operator), qh (FP8 + scales)
    backward:  dy --row+col quant--> DGrad W_d^T --> dh ;  WGrad(dy^T, qh^T) --> dW_d
               (gu, dh) --SiLU*mul backward--> dgu --row+col quant--> DGrad W_gu^T --> dx ;
               WGrad(dgu^T, qx^T) --> dW_gu
"""
from __future__ import annotations

from . import binding as jet


class MlpWeights:
    """FP8 copies of the two master weights: (q, s, qT, sT) each, as jet_quant_weight writes them."""

    def __init__(self, w_gu, w_d):
        self.inter, self.hidden = w_gu.shape[0] // 2, w_gu.shape[1]
        if tuple(w_d.shape) != (self.hidden, self.inter):
            raise ValueError("w_d must be [hidden, inter] for w_gu [2 inter, hidden]")
        self.gu = jet.quant_weight(w_gu, transposed=True)
        self.d = jet.quant_weight(w_d, transposed=True)

    def requantize(self, w_gu, w_d):
        """After an optimizer step on the bf16 masters: the same buffers are overwritten."""
        jet.quant_weight(w_gu, transposed=True, out=self.gu)
        jet.quant_weight(w_d, transposed=True, out=self.d)


def forward(x, w: MlpWeights):
    """x bf16 [M, H] -> (y bf16 [M, H], saved)."""
    I = w.inter
    qx = jet.quant_act(x)
    gu = jet.fp8_linear_fwd(qx["q_row"], qx["s_row"], w.gu[0], w.gu[1])
    qh = jet.silu_mul_quant(gu[:, :I], gu[:, I:])
    y = jet.fp8_linear_fwd(qh["q_row"], qh["s_row"], w.d[0], w.d[1])
    return y, {"qx": qx, "gu": gu, "qh": qh}


def backward(saved, dy, w: MlpWeights):
    """dy bf16 [M, H] -> dict(dx [M, H], dw_gu [2 I, H], dw_d [H, I]) in bf16, plus the
    intermediate tensors (for tests)."""
    I = w.inter
    qx, gu, qh = saved["qx"], saved["gu"], saved["qh"]
    qdy = jet.quant_act(dy, row=True, col=True)
    dh = jet.fp8_linear_dgrad(qdy["q_row"], qdy["s_row"], w.d[2], w.d[3])
    qhT = jet.quant_act(qh["q_row"], qh["s_row"], row=False, col=True)
    dw_d = jet.fp8_linear_wgrad(qdy["q_colT"], qdy["s_colT"], qhT["q_colT"], qhT["s_colT"])
    dgu = jet.silu_mul_bwd(gu[:, :I], gu[:, I:], dh)
    qdgu = jet.quant_act(dgu, row=True, col=True)
    dx = jet.fp8_linear_dgrad(qdgu["q_row"], qdgu["s_row"], w.gu[2], w.gu[3])
    qxT = jet.quant_act(qx["q_row"], qx["s_row"], row=False, col=True)
    dw_gu = jet.fp8_linear_wgrad(qdgu["q_colT"], qdgu["s_colT"], qxT["q_colT"], qxT["s_colT"])
    return {"dx": dx, "dw_gu": dw_gu, "dw_d": dw_d, "qdy": qdy, "dh": dh, "qhT": qhT, "dgu": dgu,
            "qdgu": qdgu, "qxT": qxT}


def saved_bytes(M: int, hidden: int, inter: int) -> dict:
    """Bytes kept between forward and backward per block, against saving the same tensors in bf16."""
    fp8 = lambda rows, cols: rows * cols + 4 * rows * (cols // 128)
    ours = fp8(M, hidden) + 2 * M * 2 * inter + fp8(M, inter)
    bf16 = 2 * M * hidden + 2 * M * 2 * inter + 2 * M * inter
    return {"fp8_saved": ours, "bf16_saved": bf16, "ratio": ours / bf16}
