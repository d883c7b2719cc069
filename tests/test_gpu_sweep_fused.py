"""mpq_calibrate_quant_error_rows_batch: row and tensor maxima and the per-row error sums from one
read, against the oracle and, bit for bit, against the two separate batched calls."""
import numpy as np
import pytest

import oracle
from paper_2302_01382_amd import mpq
from tests.test_gpu_sweep_batch import SHAPES, _dev, _tensors

pytestmark = pytest.mark.gpu

# also rows that do not fit the registers of their lane group (16 lanes: more than 1024 columns; a
# wave: more than 4096) and ragged ones
MORE = [(21, 1028), (9, 4100), (3, 8192), (130, 1024), (70, 4096), (17, 12)]


@pytest.mark.parametrize("b_lo,b_hi", [(2, 8), (4, 6), (2, 2)])
def test_one_read_gives_the_maxima_and_the_row_sums_of_the_two_calls(b_lo, b_hi):
    xs = _tensors(61, SHAPES + MORE)
    dx = [_dev(x) for x in xs]
    ref = mpq.sweep_plan_build(dx, b_lo, b_hi)
    mpq.calibrate_absmax_batch(ref)
    mpq.quant_error_batch(ref, mpq.PER_ROW)
    plan = mpq.sweep_plan_build(dx, b_lo, b_hi)
    for t in (plan.absmax_row_all, plan.absmax_tensor_all):
        t.fill_(-1.0)
    plan.sse_row_all.fill_(-1.0)
    mpq.calibrate_quant_error_rows_batch(plan)
    for i, x in enumerate(xs):
        am_r = oracle.absmax(x, oracle.PER_ROW)
        np.testing.assert_array_equal(plan.absmax_row[i].cpu().numpy(), am_r)
        np.testing.assert_array_equal(plan.absmax_tensor[i].cpu().numpy(), oracle.absmax(x))
        got = plan.sse_row[i].cpu().numpy()
        np.testing.assert_allclose(got, oracle.quant_error(x, am_r, b_lo, b_hi, oracle.PER_ROW), rtol=1e-4, atol=1e-30)
        np.testing.assert_array_equal(got, ref.sse_row[i].cpu().numpy())
    # the per-tensor sums then need nothing but the second call
    mpq.quant_error_batch(plan, mpq.PER_TENSOR)
    for i, x in enumerate(xs):
        np.testing.assert_allclose(plan.sse_tensor[i].cpu().numpy(), oracle.quant_error(x, oracle.absmax(x), b_lo, b_hi),
                                   rtol=1e-4, atol=1e-30)
