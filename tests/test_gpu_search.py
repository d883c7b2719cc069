"""The searches end to end: Alg. 1 / Alg. 2 from the library driving a stack evaluated with libmpq
kernels, against the oracle's searches driving the same stack evaluated with the oracle's CPU
functions.  Sizes are small enough for the oracle to run every evaluation of a search."""
import numpy as np
import pytest

import oracle
from oracle import search as osearch
from paper_2302_01382_amd import mpq, workloads
from paper_2302_01382_amd.stack import QuantStack

pytestmark = pytest.mark.gpu
BITS = [8, 4, 2]
ACT_BITS = 8


def torch():
    import torch as t
    return t


def dev(a):
    return torch().from_numpy(np.ascontiguousarray(a)).cuda()


class OracleStack:
    """The same model and score, step by step with the oracle's functions (per-output-channel
    weight scales, per-tensor activation scales, ReLU between layers)."""

    def __init__(self, x, weights):
        self.x, self.weights = x, weights
        h = x.astype(np.float32)
        for i, w in enumerate(weights):
            h = (h.astype(np.float64) @ w.astype(np.float64).T).astype(np.float32)
            if i + 1 < len(weights):
                h = np.maximum(h, np.float32(0))
        self.y_ref = h
        self.ref_norm2 = float((h.astype(np.float64) ** 2).sum())
        self.wq = []
        for w in weights:
            am = oracle.absmax(w, oracle.PER_ROW)
            per_b = {}
            for b in BITS:
                store = 4 if b <= 4 else 8
                _, codes, packed = oracle.fake_quant(w, am, b, oracle.PER_ROW, want_packed4=store == 4)
                per_b[b] = (packed if store == 4 else codes, oracle.scale_from_absmax(am, b), store)
            self.wq.append(per_b)

    def evaluate(self, bits):
        h = self.x
        for l in range(len(self.weights)):
            am = oracle.absmax(h)
            _, codes, _ = oracle.fake_quant(h, am, ACT_BITS)
            wq, sw, store = self.wq[l][bits[l]]
            y, _ = oracle.qgemm(codes, wq, oracle.scale_from_absmax(am, ACT_BITS), sw, store, oracle.PER_ROW)
            h = np.maximum(y, np.float32(0)) if l + 1 < len(self.weights) else y
        return 1.0 - oracle.sse_pair(h, self.y_ref) / self.ref_norm2


@pytest.fixture(scope="module")
def stacks():
    x, weights = workloads.search_stack(width=96, rows=160, layers=10)
    gpu = QuantStack(dev(x), [dev(w) for w in weights], BITS, ACT_BITS)
    return gpu, OracleStack(x, weights), weights


def test_reference_output_and_single_evaluations_agree(stacks):
    gpu, orc, weights = stacks
    # the fp32 reference comes from torch on one side and a float64 product on the other: close,
    # not identical; each side scores against its own
    np.testing.assert_allclose(gpu.y_ref.cpu().numpy(), orc.y_ref, rtol=2e-4, atol=1e-5)
    r = np.random.Generator(np.random.PCG64(8))
    for _ in range(12):
        bits = [int(v) for v in r.choice(BITS, len(weights))]
        a_gpu, a_orc = gpu.evaluate(bits), orc.evaluate(bits)
        # 1 - accuracy is a relative squared error; the two sides agree to the tolerance of the
        # error sums plus the difference of their reference outputs
        assert (1.0 - a_gpu) == pytest.approx(1.0 - a_orc, rel=2e-3, abs=1e-7)
    assert gpu.evaluate([8] * len(weights)) > gpu.evaluate([2] * len(weights))


def test_qe_sensitivity_matches_eq2_of_the_oracle(stacks):
    gpu, orc, weights = stacks
    for b in (2, 4, 8):
        got = gpu.qe_sensitivity(b)
        want = []
        for w in weights:
            am = oracle.absmax(w)
            want.append(oracle.eqe(oracle.quant_error(w, am, b, b)[0, 0], w.size, float(am[0])))
        np.testing.assert_allclose(got, want, rtol=1e-4)
        margins = np.diff(np.sort(want)) / np.sort(want)[:-1]
        if margins.min() > 2e-4:
            assert gpu.order_by(got) == sorted(range(len(want)), key=lambda l: (want[l], l))


@pytest.mark.parametrize("algorithm", ["bisection", "greedy"])
@pytest.mark.parametrize("target", [0.995, 0.98, 0.9, 0.7])
def test_search_result_matches_the_oracle_search(stacks, algorithm, target):
    gpu, orc, weights = stacks
    n = len(weights)
    want_s = []
    for w in weights:
        am = oracle.absmax(w)
        want_s.append(oracle.eqe(oracle.quant_error(w, am, 4, 4)[0, 0], w.size, float(am[0])))
    order = sorted(range(n), key=lambda l: (want_s[l], l))
    margins = []

    def eo(bits):
        a = orc.evaluate(bits)
        margins.append(abs(a - target))
        return a

    if algorithm == "bisection":
        want, evals_o = osearch.bisection(order, BITS, target, eo, True)
        got, evals_g = gpu.bisection(order, target, ensure_target=True)
    else:
        want, evals_o = osearch.greedy(order, BITS, target, eo)
        got, evals_g = gpu.greedy(order, target)
    # a decision is only comparable where the oracle's accuracy is clear of the target by more
    # than the two sides can differ
    if min(margins) < 2e-3 * (1.0 - target) + 1e-6:
        pytest.skip("an evaluation of this search lies within tolerance of the target: either decision is valid")
    assert got == want
    assert evals_g == evals_o
    if any(b < 8 for b in got):
        assert gpu.evaluate(got) >= target - 2e-3 * (1.0 - target)


def test_graph_replayed_evaluations_equal_eager_ones(stacks):
    """Every (layer, width) pair captured into a HIP graph and replayed several times, with eager
    evaluations in between: identical scores."""
    gpu, orc, weights = stacks
    x, _ = workloads.search_stack(width=96, rows=160, layers=10)
    graphed = QuantStack(dev(x), [dev(w) for w in weights], BITS, ACT_BITS, use_graphs=True)
    r = np.random.Generator(np.random.PCG64(9))
    for _ in range(20):
        bits = [int(v) for v in r.choice(BITS, len(weights))]
        # graph replays, eager calls from Python and the one native call: the same launches, the same bits
        assert graphed.evaluate_by_calls(bits) == gpu.evaluate_by_calls(bits) == gpu.evaluate(bits)
    assert len(graphed.graphs) == len(weights) * len(BITS)
    order = list(range(len(weights)))
    assert graphed.greedy(order, 0.9, graphed.evaluate_by_calls) == gpu.greedy(order, 0.9) == \
        gpu.greedy(order, 0.9, gpu.evaluate_by_calls)


def test_noise_sensitivity_matches_the_oracle_and_leaves_the_model_as_it_was(stacks):
    """E_N of Sec. 3.2.2 on the stack: the drop of the score when one layer's weights carry Gaussian
    noise of the spread of b-bit rounding.  The same perturbation on the oracle's side (the noise is
    bit-exact between the two), layer by layer; afterwards the model scores exactly as before."""
    gpu, orc, weights = stacks
    top = max(BITS)
    before = gpu.evaluate([top] * len(weights))
    lam, seed, b = 0.28867513, 3, 4
    got = gpu.noise_sensitivity(b, lam, seed)
    assert gpu.evaluate([top] * len(weights)) == before          # codes and step sizes restored bit for bit
    base = orc.evaluate([top] * len(weights))
    for l, w in enumerate(weights):
        am = oracle.absmax(w, oracle.PER_ROW)
        noisy = oracle.noise_inject(w, am, b, lam, seed, l, oracle.PER_ROW)
        am_n = oracle.absmax(noisy, oracle.PER_ROW)
        _, codes, _ = oracle.fake_quant(noisy, am_n, top, oracle.PER_ROW)
        keep = orc.wq[l][top]
        orc.wq[l][top] = (codes, oracle.scale_from_absmax(am_n, top), 8)
        want = base - orc.evaluate([top] * len(weights))
        orc.wq[l][top] = keep
        assert got[l] == pytest.approx(want, abs=2e-5), (l, got[l], want)
    assert max(got) > 0.0


def test_the_end_to_end_demo_runs():
    """python -m paper_2302_01382_amd.demo on a small stack: sensitivities, orders, both searches, estimates."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-m", "paper_2302_01382_amd.demo", "--layers", "4", "--width", "64", "--rows", "128"],
                       cwd=root, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout
    for needle in ("order by E_QE", "order by E_N", "order by Hessian", "bisection", "greedy", "rel.size"):
        assert needle in r.stdout, r.stdout
