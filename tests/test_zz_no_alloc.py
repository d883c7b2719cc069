"""mpq_quant_error_noalloc -- the entry point for callers that cannot allocate -- against
mpq_quant_error on the same inputs, through the C ABI: two calls in a row, the second on a smaller
input (the built-in scratch buffer still holds the first call's partial sums)."""
import numpy as np
import pytest

import oracle
from paper_2302_01382_amd import mpq

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _case(shape, seed, gran):
    import torch
    r = np.random.Generator(np.random.PCG64(seed))
    x = r.standard_normal(shape).astype(np.float32)
    dx = _dev(x)
    am = mpq.calibrate_absmax(dx, gran)
    nch = {mpq.PER_TENSOR: 1, mpq.PER_ROW: shape[0], mpq.PER_COL: shape[1]}[gran]
    out = torch.full((nch, 7), -1.0, dtype=torch.float64, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mpq.quant_error_noalloc(dx, am, out, 2, 8, gran)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before        # torch's allocator was not touched either
    want = mpq.quant_error(dx, am, 2, 8, gran)
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got, want.cpu().numpy())   # same kernels, same order: same bits
    ref = oracle.quant_error(x, am.cpu().numpy(), 2, 8, gran)
    np.testing.assert_allclose(got, ref, rtol=1e-4, atol=1e-30)


@pytest.mark.parametrize("gran", [mpq.PER_TENSOR, mpq.PER_ROW, mpq.PER_COL])
def test_two_calls_in_a_row_second_one_smaller(gran):
    # many workgroups, ragged tail (per column the partial sums grow with the columns: 2.8 of the 4 MiB)
    _case((1531, 2052) if gran != mpq.PER_COL else (1531, 1028), 41, gran)
    _case((67, 260), 42, gran)        # fewer partials than the buffer still holds from the first call


def test_long_rows_use_the_segment_partials():
    _case((9, 40000), 43, mpq.PER_ROW)   # rows longer than one segment: partial sums per segment
    _case((3, 17000), 44, mpq.PER_ROW)


def test_inputs_beyond_the_built_in_buffer_are_rejected():
    import torch
    rows, cols = 64, 1 << 20                               # per column: 64 chunks... x cols x 7 doubles
    assert mpq.quant_error_workspace_bytes(rows, cols, mpq.PER_COL) > mpq.NOALLOC_SCRATCH_BYTES
    x = torch.zeros((rows, cols), dtype=torch.float32, device="cuda")
    am = torch.ones(cols, dtype=torch.float32, device="cuda")
    out = torch.full((cols, 7), -1.0, dtype=torch.float64, device="cuda")
    with pytest.raises(mpq.MpqError) as e:
        mpq.quant_error_noalloc(x, am, out, 2, 8, mpq.PER_COL)
    assert e.value.status == mpq.ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert float(out.min()) == -1.0 and float(out.max()) == -1.0   # nothing was launched
