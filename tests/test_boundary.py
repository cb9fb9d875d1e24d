"""The C-ABI boundary without a GPU: libjet.so loads, exports every symbol that
include/jet.h declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "jet.h")


@pytest.fixture(scope="module")
def L():
    from paper_2601_14243_amd import binding
    return binding.lib()


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(jet_[a-z0-9_]+)\s*\(", src)))


def test_header_symbols_are_exported(L):
    names = _declared()
    assert {"jet_quant_act", "jet_quant_weight", "jet_fp8_linear_fwd", "jet_fp8_linear_dgrad",
            "jet_fp8_linear_wgrad", "jet_rmsnorm_quant", "jet_silu_mul_quant", "jet_silu_mul_bwd", "jet_status_str",
            "jet_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_text(L):
    from paper_2601_14243_amd import binding
    assert binding.jet_version() >= 100
    assert binding.jet_status_str(0) == "ok"
    texts = {binding.jet_status_str(i) for i in range(6)}
    assert len(texts) == 6


A = 0x1000          # a fake, 16-byte aligned, never dereferenced device address
OK, NULL, SHAPE, ALIGN, ARG = 0, 1, 2, 3, 4


def test_quant_act_argument_errors(L):
    from paper_2601_14243_amd import binding as b
    assert b.jet_quant_act(None, None, 0, 128, 128, A, A, None, None, None) == NULL
    assert b.jet_quant_act(A, None, 7, 128, 128, A, A, None, None, None) == ARG
    assert b.jet_quant_act(A, None, 1, 128, 128, A, A, None, None, None) == ARG      # FP8 source without scales
    assert b.jet_quant_act(A, None, 0, 128, 128, None, None, None, None, None) == ARG  # no output pair
    assert b.jet_quant_act(A, None, 0, 128, 128, A, None, None, None, None) == NULL   # half a pair
    assert b.jet_quant_act(A, None, 0, 128, 128, None, None, None, A, None) == NULL
    assert b.jet_quant_act(A, None, 0, 0, 128, A, A, None, None, None) == SHAPE
    assert b.jet_quant_act(A, None, 0, 4, 100, A, A, None, None, None) == SHAPE       # K % 128
    assert b.jet_quant_act(A, None, 0, 100, 128, None, None, A, A, None) == SHAPE     # M % 128 in column mode
    assert b.jet_quant_act(A + 4, None, 0, 4, 128, A, A, None, None, None) == ALIGN
    assert b.jet_quant_act(A, None, 0, 4, 128, A, A + 8, None, None, None) == ALIGN


def test_quant_weight_argument_errors(L):
    from paper_2601_14243_amd import binding as b
    assert b.jet_quant_weight(None, 128, 128, A, A, None, None, None) == NULL
    assert b.jet_quant_weight(A, 128, 128, A, None, None, None, None) == NULL
    assert b.jet_quant_weight(A, 128, 128, A, A, A, None, None) == ARG                # qT without sT
    assert b.jet_quant_weight(A, 100, 128, A, A, None, None, None) == SHAPE
    assert b.jet_quant_weight(A, 128, -128, A, A, None, None, None) == SHAPE
    assert b.jet_quant_weight(A, 128, 128, A + 2, A, None, None, None) == ALIGN


@pytest.mark.parametrize("fn", ["jet_fp8_linear_fwd", "jet_fp8_linear_dgrad", "jet_fp8_linear_wgrad"])
def test_gemm_argument_errors(L, fn):
    from paper_2601_14243_amd import binding as b
    f = getattr(b, fn)
    assert f(None, A, A, A, A, 128, 128, 128, None) == NULL
    assert f(A, A, A, A, None, 128, 128, 128, None) == NULL
    assert f(A, A, A, A, A, 0, 128, 128, None) == SHAPE
    assert f(A, A, A, A, A, 128, 100, 128, None) == SHAPE
    assert f(A, A, A, A, A, 128, 128, 200, None) == SHAPE
    assert f(A, A + 1, A, A, A, 128, 128, 128, None) == ALIGN
    want = SHAPE if fn == "jet_fp8_linear_wgrad" else None
    if want is not None:
        assert f(A, A, A, A, A, 100, 128, 128, None) == want                         # WGrad needs M % 128


def test_gemm_reduction_length_limit(L):
    """The kernels form 32-bit byte offsets from (row in tile) x (reduction length):
    a reduction axis of 2^24 or more is refused on the host."""
    from paper_2601_14243_amd import binding as b
    big = 1 << 24
    assert b.jet_fp8_linear_fwd(A, A, A, A, A, 128, 128, big, None) == SHAPE       # K
    assert b.jet_fp8_linear_dgrad(A, A, A, A, A, 128, big, 128, None) == SHAPE     # N is DGrad's reduction
    assert b.jet_fp8_linear_wgrad(A, A, A, A, A, big, 128, 128, None) == SHAPE     # M is WGrad's reduction


def test_fused_producer_argument_errors(L):
    from paper_2601_14243_amd import binding as b
    assert b.jet_rmsnorm_quant(None, A, 1e-6, 4, 128, A, A, None) == NULL
    assert b.jet_rmsnorm_quant(A, A, 1e-6, 4, 128, A, None, None) == NULL
    assert b.jet_rmsnorm_quant(A, A, -1.0, 4, 128, A, A, None) == ARG
    assert b.jet_rmsnorm_quant(A, A, float("nan"), 4, 128, A, A, None) == ARG
    assert b.jet_rmsnorm_quant(A, A, float("inf"), 4, 128, A, A, None) == ARG
    assert b.jet_rmsnorm_quant(A, A, 1e-6, 0, 128, A, A, None) == SHAPE
    assert b.jet_rmsnorm_quant(A, A, 1e-6, 4, 100, A, A, None) == SHAPE
    assert b.jet_rmsnorm_quant(A, A, 1e-6, 4, 32768 + 128, A, A, None) == SHAPE      # a row no longer fits one workgroup
    assert b.jet_rmsnorm_quant(A, A + 2, 1e-6, 4, 128, A, A, None) == ALIGN
    assert b.jet_silu_mul_quant(None, A, 128, 4, 128, A, A, None) == NULL
    assert b.jet_silu_mul_quant(A, A, 128, 4, 128, None, A, None) == NULL
    assert b.jet_silu_mul_quant(A, A, 128, 0, 128, A, A, None) == SHAPE
    assert b.jet_silu_mul_quant(A, A, 128, 4, 192, A, A, None) == SHAPE
    assert b.jet_silu_mul_quant(A, A, 64, 4, 128, A, A, None) == SHAPE               # ld < K
    assert b.jet_silu_mul_quant(A, A, 132, 4, 128, A, A, None) == SHAPE              # ld % 8
    assert b.jet_silu_mul_quant(A, A + 8, 256, 4, 128, A, A, None) == ALIGN


def test_silu_mul_bwd_argument_errors(L):
    from paper_2601_14243_amd import binding as b
    assert b.jet_silu_mul_bwd(None, A, 128, A, 4, 128, A, A, 256, None) == NULL
    assert b.jet_silu_mul_bwd(A, A, 128, None, 4, 128, A, A, 256, None) == NULL
    assert b.jet_silu_mul_bwd(A, A, 128, A, 4, 128, A, None, 256, None) == NULL
    assert b.jet_silu_mul_bwd(A, A, 128, A, 0, 128, A, A, 256, None) == SHAPE
    assert b.jet_silu_mul_bwd(A, A, 128, A, 4, 200, A, A, 256, None) == SHAPE
    assert b.jet_silu_mul_bwd(A, A, 64, A, 4, 128, A, A, 256, None) == SHAPE           # ld < K
    assert b.jet_silu_mul_bwd(A, A, 128, A, 4, 128, A, A, 100, None) == SHAPE          # ld_out < K
    assert b.jet_silu_mul_bwd(A, A, 132, A, 4, 128, A, A, 256, None) == SHAPE          # ld % 8
    assert b.jet_silu_mul_bwd(A, A, 128, A + 2, 4, 128, A, A, 256, None) == ALIGN


def test_probe_library_is_separate_and_checks_its_arguments(L):
    """The benchmark's matrix-core rate probe lives in its own library, not in the product ABI."""
    from paper_2601_14243_amd import probe as p
    assert not hasattr(L, "jet_probe_mfma_rate")
    assert p.jet_probe_mfma_rate(None, 8, 8, 0, None) == NULL
    assert p.jet_probe_mfma_rate(A, 0, 8, 0, None) == SHAPE
    assert p.jet_probe_mfma_rate(A, 8, 0, 0, None) == SHAPE
    assert p.jet_probe_mfma_rate(A, 1 << 20, 8, 0, None) == SHAPE
    assert p.jet_probe_mfma_rate(A + 4, 8, 8, 0, None) == ALIGN


def test_only_the_declared_entry_points_are_exported():
    """Built with hidden visibility: the functions in the dynamic symbol table are the jet_* entry
    points of the header and no C++ launcher (the HIP runtime's per-kernel handle objects, which
    are data, stay visible)."""
    import subprocess
    from paper_2601_14243_amd import binding
    out = subprocess.run(["nm", "-D", "--defined-only", binding._LIB_PATH], capture_output=True, text=True, check=True).stdout
    funcs = {line.split()[-1] for line in out.splitlines() if len(line.split()) == 3 and line.split()[1] in "Tt"}
    assert {f for f in funcs if not f.startswith("_")} == set(_declared()), funcs
    assert not any("launch" in f for f in funcs), funcs


def test_tile_quantizer_row_limit(L):
    from paper_2601_14243_amd import binding as b
    too_many = 65536 * 128
    assert b.jet_quant_weight(A, too_many, 128, A, A, None, None, None) == SHAPE
    assert b.jet_quant_act(A, None, 0, too_many, 128, None, None, A, A, None) == SHAPE


def test_tensor_helpers_refuse_what_the_kernels_would_read_out_of_bounds():
    """The GEMM helpers take raw pointers from torch tensors: dtype, contiguity, scale shapes,
    reduction lengths and a caller-supplied output are checked before the C call (no GPU needed:
    the checks come first)."""
    import torch
    from paper_2601_14243_amd import binding as b
    u8, f32, bf = torch.uint8, torch.float32, torch.bfloat16
    M, N, K = 4, 256, 384
    qx, sx = torch.zeros((M, K), dtype=u8), torch.ones((M, K // 128), dtype=f32)
    qw, sw = torch.zeros((N, K), dtype=u8), torch.ones((N // 128, K // 128), dtype=f32)
    for fn, args in ((b.fp8_linear_fwd, (qx, sx, qw, sw)), (b.fp8_linear_dgrad, (qx, sx, qw, sw)),
                     (b.fp8_linear_wgrad, (qw, torch.ones((N, K // 128), dtype=f32), qw, torch.ones((N, K // 128), dtype=f32)))):
        with pytest.raises(TypeError):                      # CPU tensors
            fn(*args)
    # the remaining checks are independent of the device: exercise them on a stand-in for is_cuda
    class Fake(torch.Tensor):
        @property
        def is_cuda(self):
            return True
    fake = lambda t: t.as_subclass(Fake)
    fqx, fsx, fqw, fsw = fake(qx), fake(sx), fake(qw), fake(sw)
    with pytest.raises(TypeError):
        b._need_operand(fake(qx.to(torch.int8)), fsx, 1, "qx")                     # dtype
    with pytest.raises(TypeError):
        b._need_operand(fake(torch.zeros((2 * M, K), dtype=u8)[::2]), fsx, 1, "qx")   # row-gathered, non-contiguous view
    with pytest.raises(ValueError):
        b._need_operand(fqx, fake(torch.ones((M, K // 128 + 1), dtype=f32)), 1, "qx")  # scale shape
    with pytest.raises(ValueError):
        b._need_operand(fqw, fake(torch.ones((N, K // 128), dtype=f32)), 128, "qw")    # per-row scales where blocks are due
    with pytest.raises(ValueError):
        b._need_operand(fake(torch.zeros((N, 200), dtype=u8)), fsw, 128, "qw")        # reduction not a multiple of 128
    b._need_operand(fqx, fsx, 1, "qx")
    b._need_operand(fqw, fsw, 128, "qw")
    with pytest.raises(ValueError):
        b._gemm_out(None, (M, N), fqx, fake(torch.zeros((N, K + 128), dtype=u8)), "fwd")   # K mismatch
    with pytest.raises(ValueError):
        b._gemm_out(fake(torch.zeros((M, N + 1), dtype=bf)), (M, N), fqx, fqw, "fwd")      # out shape
    with pytest.raises(TypeError):
        b._gemm_out(fake(torch.zeros((M, N), dtype=f32)), (M, N), fqx, fqw, "fwd")         # out dtype
    assert b._gemm_out(fake(torch.zeros((M, N), dtype=bf)), (M, N), fqx, fqw, "fwd").shape == (M, N)
