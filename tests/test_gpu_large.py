"""Edge case "maximum sizes": tensors with more than 2^31 elements (64-bit indexing in every
kernel) and a GEMM with more than 2^31 outputs.  The tensors are zero except for a handful of planted
values, most of them past element 2^31: zeros have code 0, error 0 and absmax 0 by definition
(Eq. 1 with x = 0), so the oracle's results on the planted values alone are the results for the
whole tensor, and elementwise outputs are checked where the oracle can compute them one by one."""
import numpy as np
import pytest

import oracle
from paper_2302_01382_amd import mpq

pytestmark = pytest.mark.gpu
ROWS, COLS = 70000, 32768          # 2,293,760,000 elements = 9.2 GB of fp32


def torch():
    import torch as t
    return t


def host(t):
    torch().cuda.synchronize()
    return t.cpu().numpy()


def test_elementwise_calls_beyond_2_31_elements():
    t = torch()
    assert ROWS * COLS > 2 ** 31
    r = np.random.Generator(np.random.PCG64(77))
    n_plant = 96
    rows = np.concatenate([r.integers(0, ROWS, n_plant - 34), r.integers(65537, ROWS, 32), [ROWS - 1, ROWS - 1]])
    cols = np.concatenate([r.integers(0, COLS, n_plant - 2), [COLS - 1, COLS - 2]])
    flat = np.unique(rows.astype(np.int64) * COLS + cols)
    rows, cols = flat // COLS, flat % COLS
    vals = r.standard_normal(flat.size).astype(np.float32)
    vals[-1] = np.float32(-3.25)                       # the maximum sits in the very last element
    assert (flat > 2 ** 31).sum() >= 30 and flat[-1] == ROWS * COLS - 1
    x = t.zeros((ROWS, COLS), dtype=t.float32, device="cuda")
    x[t.from_numpy(rows).cuda(), t.from_numpy(cols).cuda()] = t.from_numpy(vals).cuda()
    v2d = vals.reshape(1, -1)

    am = mpq.calibrate_absmax(x)
    assert host(am)[0] == oracle.absmax(v2d)[0] == np.float32(3.25)
    am_rows = host(mpq.calibrate_absmax(x, mpq.PER_ROW))
    want_rows = np.zeros(ROWS, np.float32)
    np.maximum.at(want_rows, rows, np.abs(vals))
    np.testing.assert_array_equal(am_rows, want_rows)
    am_cols = host(mpq.calibrate_absmax(x, mpq.PER_COL))
    want_cols = np.zeros(COLS, np.float32)
    np.maximum.at(want_cols, cols, np.abs(vals))
    np.testing.assert_array_equal(am_cols, want_cols)

    np.testing.assert_allclose(host(mpq.quant_error(x, am)), oracle.quant_error(v2d, host(am)), rtol=1e-4)

    for bits in (8, 3):
        _, codes, _ = mpq.fake_quant(x, am, bits, want_y=False, want_codes=True)
        _, want, _ = oracle.fake_quant(v2d, host(am), bits)
        got = host(codes[t.from_numpy(rows).cuda(), t.from_numpy(cols).cuda()])
        np.testing.assert_array_equal(got, want.ravel())
        assert int(t.count_nonzero(codes).item()) == int(np.count_nonzero(want))
        del codes

    # noise: element i of the stream is group i // 4, lane i % 4, also past 2^31
    lam, seed, sid = 0.28867513, 11, 3
    y = mpq.noise_inject(x, am, 4, lam, seed, sid)
    sigma = np.float32(np.float32(lam) * oracle.scale_from_absmax(host(am), 4)[0])
    probe = np.concatenate([flat, [0, 5, 2 ** 31 - 1, 2 ** 31, 2 ** 31 + 6, ROWS * COLS - 3]])
    xs = np.zeros(probe.size, np.float32)
    xs[:flat.size] = vals
    want = np.array([np.float32(np.float64(sigma) * np.float64(oracle.gauss4(seed, sid, int(i) // 4)[int(i) % 4]) + np.float64(xv))
                     for i, xv in zip(probe, xs)], np.float32)
    got = host(y.view(-1)[t.from_numpy(probe).cuda()])
    np.testing.assert_array_equal(got, want)


def test_qgemm_beyond_2_31_outputs_on_sampled_rows():
    t = torch()
    M, N, K = 1_100_000, 2048, 64
    assert M * N > 2 ** 31
    g = t.Generator(device="cuda")
    g.manual_seed(5)
    a = t.randint(-127, 128, (M, K), dtype=t.int8, device="cuda", generator=g)
    w = t.randint(-127, 128, (N, K), dtype=t.int8, device="cuda", generator=g)
    r = np.random.Generator(np.random.PCG64(6))
    sa = np.array([0.003], np.float32)
    sw = (r.random(N).astype(np.float32) + 0.5) * np.float32(1e-3)
    dsa, dsw = t.from_numpy(sa).cuda(), t.from_numpy(sw).cuda()
    y, _ = mpq.qgemm(a, w, dsa, dsw, 8, mpq.PER_ROW)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, M - 257, M - 256, M - 2, M - 1], r.integers(0, M, 40),
                                     r.integers((2 ** 31) // N + 1, M, 40)]))
    idx = t.from_numpy(rows).cuda()
    y_o, _ = oracle.qgemm(host(a[idx]), host(w), sa, sw, 8, oracle.PER_ROW)
    np.testing.assert_allclose(host(y[idx]), y_o, rtol=1e-5, atol=0)
    # the score epilogue over the same outputs: against a reference that differs in sampled rows only
    y_ref = y.clone()
    y_ref[idx] += 1.0
    sse, _ = mpq.qgemm_score(a, w, dsa, dsw, y_ref, 8, mpq.PER_ROW)
    assert host(sse)[0] == pytest.approx(rows.size * N, rel=1e-4)
