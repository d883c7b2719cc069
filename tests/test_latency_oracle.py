"""Pins of the oracle's deployment estimates (oracle/latency.py) against the figures the paper
prints in Table 1, and the library's host functions against the oracle.  CPU only."""
import os

import numpy as np
import pytest

from oracle import latency as olat

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_uniform_precision_baselines.txt")


def rows():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        out[(f[0], f[1])] = [float(v) for v in f[2:]]
    return out


def test_relative_latency_reproduces_the_printed_percentages():
    """A model whose every layer runs at one precision has the latency the table prints for that
    precision; relative to the 16-bit model that is the printed percentage (two decimals)."""
    for model in ("ResNet50", "BERT"):
        l4, l8, l16, r4, r8, r16 = rows()[(model, "latency_ms")]
        kernel = [{4: l4, 8: l8, 16: l16}]                     # the whole model as one kernel
        for b, want in ((4, r4), (8, r8), (16, r16)):
            assert round(100.0 * olat.relative_latency(kernel, [b], 16), 2) == pytest.approx(want, abs=0.006)
        # split the same latencies over several layers in any proportion: the sum does not care
        parts = [0.2, 0.5, 0.3]
        kernel3 = [{b: p * v for b, v in kernel[0].items()} for p in parts]
        assert olat.model_latency(kernel3, [8, 8, 8]) == pytest.approx(l8, rel=1e-12)
        mixed = olat.model_latency(kernel3, [4, 16, 8])
        assert mixed == pytest.approx(0.2 * l4 + 0.5 * l16 + 0.3 * l8, rel=1e-12)
        assert l4 < mixed < l16


def test_model_size_reproduces_the_printed_megabytes():
    for model in ("ResNet50", "BERT"):
        s4, s8, s16, r4, r8, r16 = rows()[(model, "size_MB")]
        params = int(round(s16 * 1e6 / 2))                      # 16-bit model: two bytes per parameter
        for b, size, rel in ((4, s4, r4), (8, s8, r8), (16, s16, r16)):
            assert olat.model_size_bytes([params], [b]) / 1e6 == pytest.approx(size, abs=0.006)
            assert 100.0 * olat.relative_size([params], [b], 16) == pytest.approx(rel, abs=1e-9)
        # parameters split over layers with different widths
        p = [params // 4, params // 2, params - params // 4 - params // 2]
        assert olat.model_size_bytes(p, [4, 8, 16]) == p[0] / 2 + p[1] + 2 * p[2]


def test_library_estimates_match_the_oracle():
    from paper_2302_01382_amd import mpq
    r = np.random.Generator(np.random.PCG64(80))
    n_layers, widths = 9, [8, 4, 2]
    table = r.random((n_layers, len(widths))) * 20 + 1
    kernel = [{b: table[l, i] for i, b in enumerate(widths)} for l in range(n_layers)]
    params = [int(v) for v in r.integers(1000, 10 ** 7, n_layers)]
    for _ in range(20):
        idx = [int(v) for v in r.integers(0, len(widths), n_layers)]
        bits = [widths[i] for i in idx]
        assert mpq.latency_estimate(table, idx) == pytest.approx(olat.model_latency(kernel, bits), rel=1e-14)
        assert mpq.model_size_bytes(params, bits) == pytest.approx(olat.model_size_bytes(params, bits), rel=1e-14)
    L = mpq.lib()
    out = mpq.C.c_double()
    t = np.ascontiguousarray(table)
    bad = (mpq.C.c_int * n_layers)(*([0] * (n_layers - 1) + [3]))
    assert L.mpq_latency_estimate(t.ctypes.data, n_layers, 3, bad, mpq.C.byref(out)) == mpq.ERR_SHAPE
    assert L.mpq_latency_estimate(None, n_layers, 3, bad, mpq.C.byref(out)) == mpq.ERR_NULL
