"""The latency / footprint estimate (sum of per-layer kernel latencies, parameters x bits): host
arithmetic checked on a table written by hand; the measured table itself on the GPU."""
import pytest

from paper_2302_01382_amd import latency as lat

LAYERS = [(1, 1024, 4096), (1, 4096, 1024), (1, 1024, 1024)]
TABLE = lat.LatencyTable({(1, 1024, 4096, 8): 10.0, (1, 1024, 4096, 4): 6.0, (1, 4096, 1024, 8): 9.0,
                          (1, 4096, 1024, 4): 5.5, (1, 1024, 1024, 8): 4.0, (1, 1024, 1024, 4): 3.0})


def test_estimate_is_the_sum_of_the_layers_kernel_latencies():
    assert TABLE.estimate_us(LAYERS, [8, 8, 8]) == 23.0
    assert TABLE.estimate_us(LAYERS, [4, 8, 2]) == 6.0 + 9.0 + 3.0     # 2-bit weights travel as int4
    assert TABLE.relative(LAYERS, [4, 4, 4]) == pytest.approx(14.5 / 23.0)
    assert TABLE.relative(LAYERS, [8, 8, 8]) == 1.0
    with pytest.raises(ValueError):
        TABLE.estimate_us(LAYERS, [8, 8])
    with pytest.raises(KeyError):
        TABLE.lookup((2, 2, 2), 8)


def test_footprint_is_parameters_times_bits():
    p = [k * n for _, k, n in LAYERS]
    assert lat.footprint_bytes(LAYERS, [8, 4, 2]) == p[0] + p[1] / 2 + p[2] / 4
    assert lat.relative_footprint(LAYERS, [4, 4, 4]) == 0.5
    assert lat.storage_bits(2) == 4 and lat.storage_bits(4) == 4 and lat.storage_bits(5) == 8


@pytest.mark.gpu
def test_measured_table_on_the_gpu():
    shapes = [(1, 1024, 4096), (384, 1024, 1024)]
    t = lat.LatencyTable().measure(shapes, reps=10, warmup=2)
    assert set(t.us) == {(m, k, n, s) for (m, k, n) in shapes for s in (8, 4)}
    assert all(0.5 < v < 5000.0 for v in t.us.values())
    # at batch one the layer streams its weights once: half the bytes must not cost more time
    assert t.us[(1, 1024, 4096, 4)] <= 1.15 * t.us[(1, 1024, 4096, 8)]
    assert t.estimate_us(shapes, [8, 4]) == t.us[(1, 1024, 4096, 8)] + t.us[(384, 1024, 1024, 4)]
