"""Packed int4 weights must not make the quantized layer slower than int8 weights of the same shape:
the paper's latency model (experiments section, "Compute Latency Estimates": one kernel latency per
layer and precision) only rewards a lower precision if its kernel is at least as fast.  A timing
test, so it is generous (12 %, best of five runs of 20 launches) and collected late: what it guards
against is a structural regression such as bank-conflicted reads of the packed tile, which cost
5-15 %.  Operands are cold (rotated through more buffers than the memory-side cache holds), as a
layer's weights are when inference reaches it: that is the latency the table is made of."""
import pytest

from paper_2302_01382_amd import latency as lat

pytestmark = pytest.mark.gpu

# one shape per tile size of the fast path, plus a batch-1 shape that is split along K
SHAPES = [(16384, 4096, 1024), (12288, 3072, 768), (6272, 1024, 1024), (1568, 4608, 512), (49, 4608, 512)]


@pytest.mark.parametrize("mkn", SHAPES)
def test_packed_int4_weights_are_not_slower(mkn):
    M, K, N = mkn
    best = {}
    for st in (8, 4):
        best[st] = min(lat.time_qgemm(M, K, N, st, reps=20, warmup=3) for _ in range(5))
    assert best[4] <= 1.12 * best[8], "W4 %.2f us against W8 %.2f us" % (best[4], best[8])
