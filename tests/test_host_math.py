"""The library's host-side steps (Eq. 2's normalisation, the trace estimate's mean and standard
error) against the oracle's, and the Python model wrapper's use of them.  No GPU needed: these are
host functions of libmpq on host values."""
import math

import numpy as np
import pytest

import oracle
from paper_2302_01382_amd import mpq


def test_eqe_matches_the_oracle():
    r = np.random.Generator(np.random.PCG64(70))
    for _ in range(50):
        sse, n, m = float(r.random() * 10), int(r.integers(1, 10 ** 6)), float(np.float32(r.random() * 3 + 1e-3))
        assert mpq.eqe(sse, n, m) == pytest.approx(oracle.eqe(sse, n, m), rel=1e-15)
    assert mpq.eqe(1.0, 10, 0.0) == 0.0 and oracle.eqe(1.0, 10, 0.0) == 0.0     # all-zero tensor
    assert mpq.eqe(1.0, 0, 1.0) == 0.0
    # from real sums: a tensor swept by the oracle
    x = r.standard_normal((40, 50)).astype(np.float32)
    m = oracle.absmax(x)
    for s in oracle.quant_error(x, m)[0]:
        assert mpq.eqe(s, x.size, float(m[0])) == pytest.approx(oracle.eqe(s, x.size, float(m[0])), rel=1e-15)


def test_eqe_channels_matches_the_oracle():
    r = np.random.Generator(np.random.PCG64(71))
    x = (r.standard_normal((17, 64)) * np.linspace(0.2, 2.0, 17)[:, None]).astype(np.float32)
    x[5] = 0.0
    for gran, nch in ((oracle.PER_ROW, 17), (oracle.PER_COL, 64)):
        m = oracle.absmax(x, gran)
        for lo, hi in ((2, 8), (4, 4), (3, 6)):
            sse = oracle.quant_error(x, m, lo, hi, gran)
            np.testing.assert_allclose(mpq.eqe_channels(sse, x.size, m), oracle.eqe_channels(sse, x.size, m), rtol=1e-15)
    L = mpq.lib()
    out = (mpq.C.c_double * 7)()
    assert L.mpq_eqe_channels(None, None, 1, 7, 1, out) == mpq.ERR_NULL
    one = np.zeros((1, 7))
    am = np.ones(1, np.float32)
    assert L.mpq_eqe_channels(one.ctypes.data, am.ctypes.data, 0, 7, 1, out) == mpq.ERR_SHAPE
    assert L.mpq_eqe_channels(one.ctypes.data, am.ctypes.data, 1, 8, 1, out) == mpq.ERR_BITS


def test_hutchinson_trace_matches_the_oracle():
    r = np.random.Generator(np.random.PCG64(72))
    x = r.standard_normal((33, 20)).astype(np.float32)
    for probes in (1, 2, 16):
        v = oracle.rademacher(3, 1, probes, 20)
        q = oracle.hutchinson_quad(x, v)
        est, err = mpq.hutchinson_trace(q, x.shape[0])
        est_o, err_o = oracle.hutchinson_trace(x, v)
        assert est == pytest.approx(est_o, rel=1e-14)
        if probes == 1:
            assert math.isnan(err) and math.isnan(err_o)
        else:
            assert err == pytest.approx(err_o, rel=1e-12)
    L = mpq.lib()
    e = mpq.C.c_double()
    assert L.mpq_hutchinson_trace(None, 4, 4, mpq.C.byref(e), None) == mpq.ERR_NULL
    q = np.ones(4)
    assert L.mpq_hutchinson_trace(q.ctypes.data, 0, 4, mpq.C.byref(e), None) == mpq.ERR_SHAPE
    assert L.mpq_hutchinson_trace(q.ctypes.data, 4, 8, mpq.C.byref(e), None) == mpq.OK and e.value == 0.25
