"""The batched sensitivity sweep (mpq_calibrate_absmax_batch, mpq_quant_error_batch) against the CPU
oracle tensor by tensor, and against the single-tensor calls of the library."""
import numpy as np
import pytest

import oracle
from paper_2302_01382_amd import mpq

pytestmark = pytest.mark.gpu
RTOL_SSE = 1e-4

# rows x cols: short rows (16 lanes per row), long rows (a wave per row), ragged row counts, a tensor
# smaller than one chunk, one of several chunks with a ragged last chunk, a single row
SHAPES = [(37, 260), (300, 1024), (5, 4096), (129, 2052), (1, 4), (64, 16384), (1000, 516), (33, 2048)]


def _tensors(seed, shapes=SHAPES):
    r = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i, s in enumerate(shapes):
        x = (r.standard_normal(s) * (0.02 * (1 + i))).astype(np.float32)
        if x.size > 100:
            x.ravel()[r.integers(0, x.size, 3)] *= np.float32(9.0)     # a few outliers
        out.append(x)
    out[1][7, :] = 0.0                                                 # an all-zero channel
    return out


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_batched_calibration_is_exact():
    xs = _tensors(51)
    plan = mpq.sweep_plan_build([_dev(x) for x in xs])
    mpq.calibrate_absmax_batch(plan)
    for i, x in enumerate(xs):
        np.testing.assert_array_equal(plan.absmax_row[i].cpu().numpy(), oracle.absmax(x, oracle.PER_ROW))
        np.testing.assert_array_equal(plan.absmax_tensor[i].cpu().numpy(), oracle.absmax(x))


@pytest.mark.parametrize("b_lo,b_hi", [(2, 8), (3, 5), (8, 8)])
def test_batched_error_sums_match_the_oracle_and_the_single_calls(b_lo, b_hi):
    xs = _tensors(52)
    dx = [_dev(x) for x in xs]
    plan = mpq.sweep_plan_build(dx, b_lo, b_hi)
    mpq.calibrate_absmax_batch(plan)
    mpq.quant_error_batch(plan, mpq.PER_TENSOR)
    mpq.quant_error_batch(plan, mpq.PER_ROW)
    got_t = [s.cpu().numpy().copy() for s in plan.sse_tensor]
    got_r = [s.cpu().numpy().copy() for s in plan.sse_row]
    for i, x in enumerate(xs):
        am_t, am_r = oracle.absmax(x), oracle.absmax(x, oracle.PER_ROW)
        np.testing.assert_allclose(got_t[i], oracle.quant_error(x, am_t, b_lo, b_hi), rtol=RTOL_SSE, atol=1e-30)
        np.testing.assert_allclose(got_r[i], oracle.quant_error(x, am_r, b_lo, b_hi, oracle.PER_ROW),
                                   rtol=RTOL_SSE, atol=1e-30)
        # per row the batch walks a row exactly as the single-tensor call does: same bits
        single = mpq.quant_error(dx[i], plan.absmax_row[i], b_lo, b_hi, mpq.PER_ROW).cpu().numpy()
        np.testing.assert_array_equal(got_r[i], single)
    # both granularities from one read: the same per-row bits, the per-tensor sums to tolerance
    plan.sse_tensor_all.fill_(-1.0)
    plan.sse_row_all.fill_(-1.0)
    mpq.quant_error_batch(plan, mpq.SWEEP_TENSOR_AND_ROW)
    for i, x in enumerate(xs):
        np.testing.assert_array_equal(plan.sse_row[i].cpu().numpy(), got_r[i])
        np.testing.assert_allclose(plan.sse_tensor[i].cpu().numpy(), oracle.quant_error(x, oracle.absmax(x), b_lo, b_hi),
                                   rtol=RTOL_SSE, atol=1e-30)
    # reproducible: fixed combination order
    again = mpq.quant_error_batch(plan, mpq.SWEEP_TENSOR_AND_ROW).sse_tensor_all.cpu().numpy().copy()
    np.testing.assert_array_equal(again, mpq.quant_error_batch(plan, mpq.SWEEP_TENSOR_AND_ROW).sse_tensor_all.cpu().numpy())


def test_batched_sweep_of_a_set_lying_on_the_grid_is_zero():
    r = np.random.Generator(np.random.PCG64(53))
    xs = []
    for b in (2, 4, 8):
        q = (1 << (b - 1)) - 1
        codes = r.integers(-q, q + 1, size=(70, 1028))
        codes[:, 0] = q                                   # every row attains the maximum
        xs.append((codes * np.float32(2.0 ** -6)).astype(np.float32))
    plan = mpq.sweep_plan_build([_dev(x) for x in xs])
    mpq.calibrate_absmax_batch(plan)
    mpq.quant_error_batch(plan, mpq.SWEEP_TENSOR_AND_ROW)
    for i, b in enumerate((2, 4, 8)):
        assert float(plan.sse_tensor[i][0, b - 2]) == 0.0
        assert float(plan.sse_row[i][:, b - 2].abs().max()) == 0.0


def test_batched_sweep_and_noalloc_call_replay_in_a_hip_graph():
    """The calls only enqueue kernels (no memset nodes, no allocation), so a captured sweep replays:
    three replays with eager work and synchronisations between them, every replay checked against
    the eager result on fresh data written into the same tensors."""
    import torch
    xs = _tensors(54)
    dx = [_dev(x) for x in xs]
    plan = mpq.sweep_plan_build(dx)
    big = dx[6]                                              # 1000 x 516
    am_big = torch.empty(1, dtype=torch.float32, device="cuda")
    out_na = torch.empty((1, 7), dtype=torch.float64, device="cuda")
    ws = mpq.Workspace()
    ws.get(1 << 20)

    def sweep():
        mpq.calibrate_absmax_batch(plan)
        mpq.quant_error_batch(plan, mpq.PER_TENSOR)
        mpq.quant_error_batch(plan, mpq.PER_ROW)
        mpq.calibrate_absmax(big, out=am_big, ws=ws)
        mpq.quant_error_noalloc(big, am_big, out_na)

    sweep()                                                  # sizes every workspace before the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sweep()
    r = np.random.Generator(np.random.PCG64(55))
    for it in range(3):
        for t in dx:                                         # new values in place: the graph holds addresses only
            t.copy_(torch.from_numpy((r.standard_normal(tuple(t.shape)) * (it + 1)).astype(np.float32)))
        plan.sse_tensor_all.fill_(-1.0)
        plan.sse_row_all.fill_(-1.0)
        out_na.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        got = (plan.sse_tensor_all.clone(), plan.sse_row_all.clone(), plan.absmax_row_all.clone(), out_na.clone())
        sweep()                                              # the same, eagerly
        torch.cuda.synchronize()
        want = (plan.sse_tensor_all, plan.sse_row_all, plan.absmax_row_all, out_na)
        for a, b in zip(got, want):
            assert torch.equal(a, b)
        assert float(out_na.min()) >= 0.0
        # and against the oracle, once per replay, on one tensor
        x6 = big.cpu().numpy()
        np.testing.assert_allclose(got[3].cpu().numpy(), oracle.quant_error(x6, oracle.absmax(x6)), rtol=RTOL_SSE)
