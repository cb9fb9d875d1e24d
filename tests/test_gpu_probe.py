"""The matrix-core rate probe (a measurement aid of the benchmark, not a step of the
layer): it runs, writes one value per wave, and with all-zero operands that value is 0."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jet():
    from paper_2601_14243_amd import probe as j
    assert torch.cuda.is_available()
    j.lib()
    return j


def test_probe_runs_and_zero_data_sums_to_zero(jet):
    wgs, iters = 64, 50
    out = torch.full((wgs * 8,), 7.0, dtype=torch.float32, device="cuda")
    st = jet.jet_probe_mfma_rate(out.data_ptr(), wgs, iters, 1, torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    assert torch.count_nonzero(out).item() == 0
    st = jet.jet_probe_mfma_rate(out.data_ptr(), wgs, iters, 0, torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and torch.count_nonzero(out).item() > wgs * 4


def test_probe_rate_is_positive(jet):
    rate = jet.probe_mfma_rate(workgroups=256, iters=200, zero_data=True, repeats=2)
    assert rate > 1e12   # any working matrix core exceeds 1 TFLOP/s by orders of magnitude
