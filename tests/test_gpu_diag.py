"""The measurement aids mpq_diag_mfma_rate and mpq_diag_sweep_alu_rate: they run, and report plausible rates."""
import pytest

from paper_2302_01382_amd import mpq

pytestmark = pytest.mark.gpu


def test_mfma_rate_is_plausible_and_data_dependent():
    import torch
    n = mpq.diag_mfma_operand_bytes()
    const = torch.full((n,), 3, dtype=torch.int8, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(3)
    rnd = torch.randint(-127, 128, (n,), dtype=torch.int8, device="cuda", generator=g)
    r_const, r_rnd = mpq.diag_mfma_rate(const, iters=512), mpq.diag_mfma_rate(rnd, iters=512)
    assert 1000.0 < r_rnd <= 5100.0 and 1000.0 < r_const <= 5100.0      # TOP/s; nominal peak 5000
    with pytest.raises(mpq.MpqError):
        mpq.diag_mfma_rate(const[: n // 2])


def test_sweep_alu_rate_is_plausible():
    r = mpq.diag_sweep_alu_rate(iters=200)
    # T lane-op/s: 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz = 78.6 is the fp32 vector peak
    assert 15.0 < r <= 80.0
    with pytest.raises(mpq.MpqError):
        mpq.diag_sweep_alu_rate(iters=0)
