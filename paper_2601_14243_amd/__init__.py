"""MI355X-native block-scaled FP8 linear layer (Jet-RL's unified precision flow).

The product is ``libjet.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/jet.h``); this package is a thin ctypes binding with the same names.
PyTorch supplies device memory and streams only.
"""
from .binding import (JET_SRC_BF16, JET_SRC_FP8_ROW, JetError, fp8_linear_dgrad, fp8_linear_fwd,
                      fp8_linear_wgrad, jet_fp8_linear_dgrad, jet_fp8_linear_fwd,
                      jet_fp8_linear_wgrad, jet_quant_act, jet_quant_weight, jet_status_str,
                      jet_version, lib, quant_act, quant_weight,
                      jet_rmsnorm_quant, jet_silu_mul_quant, rmsnorm_quant, silu_mul_quant,
                      jet_silu_mul_bwd, silu_mul_bwd)

__all__ = [
    "JET_SRC_BF16", "JET_SRC_FP8_ROW", "JetError", "lib", "jet_version", "jet_status_str",
    "jet_quant_act", "jet_quant_weight", "jet_fp8_linear_fwd", "jet_fp8_linear_dgrad",
    "jet_fp8_linear_wgrad", "quant_act", "quant_weight", "fp8_linear_fwd", "fp8_linear_dgrad",
    "fp8_linear_wgrad", "jet_rmsnorm_quant",
    "jet_silu_mul_quant", "rmsnorm_quant", "silu_mul_quant", "jet_silu_mul_bwd", "silu_mul_bwd",
]
