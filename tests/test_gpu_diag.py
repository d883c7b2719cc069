"""The measurement aid mpq_diag_mfma_rate: runs, and reports a plausible int8 matrix rate."""
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
