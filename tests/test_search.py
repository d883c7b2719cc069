"""Alg. 1 (bisection) and Alg. 2 (greedy): the oracle against hand traces, closed forms and
invariants, and the library's host code against the oracle.  No GPU involved."""
import math
import os

import numpy as np
import pytest

from oracle import search as osearch
from paper_2302_01382_amd import mpq

HERE = os.path.dirname(os.path.abspath(__file__))


def count_at(bits, b):
    return sum(1 for v in bits if v == b)


def at_most(k, b, log=None):
    """Evaluator that meets the target 1.0 iff at most k layers sit at width b."""
    def f(bits):
        if log is not None:
            log.append(list(bits))
        return 1.0 if count_at(bits, b) <= k else 0.0
    return f


# ------------------------------------------------------------------------------ oracle pins
def read_traces():
    rows = []
    for line in open(os.path.join(HERE, "golden", "bisection_hand_traces.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, seq, printed, safe = [p.strip() for p in line.split("|")]
        n, k = map(int, head.split())
        rows.append((n, k, [int(s[:-1]) for s in seq.split()], int(printed), int(safe)))
    return rows


def pass_at_4_on_a_list_of(n, k, ensure, search=osearch.bisection):
    """Runs widths (16, 4) on n + 1 layers.  Every evaluation of the pass at 16 meets the target
    (nothing sits at 4 yet), which by the update rules leaves the first n layers in the list; the
    pass at 4 then works on a list of exactly n.  Returns (thresholds that pass evaluated, w)."""
    _, evals_16 = search(list(range(n + 1)), [16], 1.0, lambda bits: 1.0)
    log = []
    w, evals = search(list(range(n + 1)), [16, 4], 1.0, at_most(k, 4, log), ensure)
    assert evals == len(log)
    return [count_at(bits, 4) for bits in log[evals_16:]], w


@pytest.mark.parametrize("n,k,seq,printed,safe", read_traces())
def test_oracle_bisection_follows_the_hand_traces(n, k, seq, printed, safe):
    for ensure, want in ((False, printed), (True, safe)):
        thresholds, w = pass_at_4_on_a_list_of(n, k, ensure)
        assert thresholds == seq
        assert w == [4] * want + [16] * (n + 1 - want)


def test_oracle_bisection_closed_form_on_monotone_evaluators():
    """With the fall-back, bisection on "at most k layers may go to b" returns exactly
    min(k, len - 1): the largest admissible count the floor arithmetic can reach (thr never gets
    to len).  Evaluations per width stay within ceil(log2 len) + 1."""
    for n in range(1, 70):
        for k in range(0, n + 1):
            thresholds, w = pass_at_4_on_a_list_of(n, k, True)
            want = min(k, n - 1)
            assert w == [4] * want + [16] * (n + 1 - want)
            assert len(thresholds) <= math.ceil(math.log2(max(n, 2))) + 1
            # as printed the result is that count or, after a closing miss, one more
            _, w_printed = pass_at_4_on_a_list_of(n, k, False)
            assert count_at(w_printed, 4) in (want, want + 1)


def test_oracle_bisection_only_lowers_prefixes_and_shrinks_the_list():
    r = np.random.Generator(np.random.PCG64(1))
    for trial in range(50):
        n = int(r.integers(1, 30))
        order = [int(v) for v in r.permutation(n)]
        caps = {8: int(r.integers(0, n + 1)), 4: int(r.integers(0, n + 1)), 2: int(r.integers(0, n + 1))}
        log = []

        def ev(bits):
            log.append(list(bits))
            return 1.0 if all(sum(1 for v in bits if v <= b) <= caps[b] for b in caps) else 0.0

        w, evals = osearch.bisection(order, [16, 8, 4, 2], 1.0, ev, True)
        assert evals == len(log)
        for bits in log + [w]:
            by_order = [bits[l] for l in order]
            assert by_order == sorted(by_order)   # widths never decrease along the sensitivity order
        if any(v < 16 for v in w):
            assert ev(w) == 1.0                   # with the fall-back the answer meets the target


def test_oracle_greedy_closed_form_on_separable_evaluators():
    """If the model meets the target iff every layer l keeps at least need[l] bits, Alg. 2 must end
    with the smallest listed width >= need[l] for every layer, after trying each layer at one
    width more than it could take (or at all of them)."""
    r = np.random.Generator(np.random.PCG64(2))
    bs = [16, 8, 4, 2]
    for trial in range(100):
        n = int(r.integers(1, 25))
        need = [int(v) for v in r.integers(1, 17, n)]
        order = [int(v) for v in r.permutation(n)]
        w, evals = osearch.greedy(order, bs, 1.0, lambda bits: 1.0 if all(b >= m for b, m in zip(bits, need)) else 0.0)
        assert w == [min(b for b in bs if b >= m) for m in need]
        assert evals == sum(min(len(bs), 1 + sum(1 for b in bs if b >= m)) for m in need)


def test_oracle_greedy_budget_evaluator_invariants():
    """A non-separable evaluator (error budget shared by all layers): every accepted step was
    evaluated and met the target, so the answer does; layers early in the order are served first."""
    r = np.random.Generator(np.random.PCG64(3))
    for trial in range(50):
        n = int(r.integers(2, 20))
        cost = r.random(n) + 0.1
        budget = float(r.random() * n * 0.05)

        def ev(bits):
            return -float(sum(c * 4.0 ** (-b) for c, b in zip(cost, bits)) * 4.0 ** 4)

        order = list(range(n))
        w, evals = osearch.greedy(order, [8, 4, 2], -budget, ev)
        assert evals <= 3 * n
        if w != [8] * n or ev(w) >= -budget:
            assert ev(w) >= -budget
        # identical layers: the one that comes first in the order is never left at more bits
        cost[:] = 1.0
        w, _ = osearch.greedy(order, [8, 4, 2], -budget, ev)
        assert w == sorted(w)


# --------------------------------------------------------------------- library vs oracle
def random_evaluator(r, n):
    kind = int(r.integers(0, 3))
    if kind == 0:      # shared error budget
        cost = r.random(n) + 0.05
        return (lambda bits: -float(sum(c * 4.0 ** (8 - b) for c, b in zip(cost, bits)))), -float(r.random() * n * 8)
    if kind == 1:      # per-layer minimum
        need = r.integers(1, 10, n)
        return (lambda bits: 1.0 if all(b >= m for b, m in zip(bits, need)) else 0.0), 1.0
    table = {}         # arbitrary but deterministic: a hash of the configuration
    seed = int(r.integers(0, 1 << 30))

    def f(bits):
        key = tuple(bits)
        if key not in table:
            table[key] = float(np.random.Generator(np.random.PCG64([seed, *key])).random())
        return table[key]
    return f, float(r.random())


@pytest.mark.parametrize("algorithm", ["bisection", "bisection_ensure", "greedy"])
def test_library_search_matches_the_oracle_call_by_call(algorithm):
    r = np.random.Generator(np.random.PCG64(4))
    for trial in range(120):
        n = int(r.integers(1, 40))
        order = [int(v) for v in r.permutation(n)]
        bs = sorted({int(v) for v in r.choice([16, 8, 6, 4, 3, 2], int(r.integers(1, 5)), replace=False)}, reverse=True)
        ev, target = random_evaluator(r, n)
        log_o, log_l = [], []

        def eo(bits):
            log_o.append(list(bits))
            return ev(bits)

        def el(bits):
            log_l.append(list(bits))
            return ev(bits)

        if algorithm == "greedy":
            want = osearch.greedy(order, bs, target, eo)
            got = mpq.search_greedy(order, bs, target, el)
        else:
            ensure = algorithm.endswith("ensure")
            want = osearch.bisection(order, bs, target, eo, ensure)
            got = mpq.search_bisection(order, bs, target, el, ensure)
        assert got == want
        assert log_l == log_o     # the same configurations, in the same order


def test_library_search_widths_in_any_order_and_validation():
    ev = at_most(2, 4)
    assert mpq.search_greedy([0, 1, 2], [4, 8], 1.0, ev) == osearch.greedy([0, 1, 2], [4, 8], 1.0, ev)
    for fn in (mpq.search_bisection, mpq.search_greedy):
        with pytest.raises(mpq.MpqError) as e:
            fn([0, 0, 1], [8, 4], 1.0, ev)           # not a permutation
        assert e.value.status == mpq.ERR_SHAPE
        with pytest.raises(mpq.MpqError) as e:
            fn([0, 1], [8, 1], 1.0, ev)
        assert e.value.status == mpq.ERR_BITS
        with pytest.raises(mpq.MpqError) as e:
            fn([], [8], 1.0, ev)
        assert e.value.status == mpq.ERR_SHAPE
    L = mpq.lib()
    assert L.mpq_search_greedy(None, 1, None, 1, 0.0, 0, mpq.EVAL_FN(lambda b, n, u: 0.0), None, None, None) == mpq.ERR_NULL


def test_library_search_reports_an_exception_of_the_evaluator():
    calls = []

    def ev(bits):
        calls.append(1)
        if len(calls) == 3:
            raise ValueError("evaluation failed")
        return 1.0

    with pytest.raises(ValueError):
        mpq.search_greedy(list(range(6)), [8, 4], 1.0, ev)
    assert len(calls) == 3    # no evaluation runs after the failure
