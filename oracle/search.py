"""Oracle for the two configuration searches (Alg. 1 bisection, Alg. 2 greedy): plain Python,
written from the paper's description in its notation (w working configuration, ll layer list
sorted by sensitivity, thr / upl / lowl threshold and its bounds, lw local configuration, ql
layers that stay quantizable).  TEST INFRASTRUCTURE ONLY: nothing on the product path may import
this module.

Readings where the paper leaves the arithmetic open (same as the product's, stated there too):
bit widths are visited in the order given; thr is an integer, halving is floor division; the
repeat loop of Alg. 1 ends when an update leaves thr as it was.  ensure_target=True is the one
documented departure: if that loop ends on an evaluation that missed the target, thr falls back
to lowl."""
from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

Evaluate = Callable[[List[int]], float]   # f(x, lw) -> accuracy a


def bisection(ll: Sequence[int], bs: Sequence[int], t: float, evaluate: Evaluate,
              ensure_target: bool = False) -> Tuple[List[int], int]:
    """Alg. 1.  ll: layer ids in ascending order of sensitivity.  Returns (w, number of evaluations)."""
    n = len(ll)
    w = [max(bs)] * n
    ll = list(ll)
    evaluations = 0
    for b in bs:
        # quantize the least sensitive part of the list, ll[0:thr], to b and move thr by halves
        thr, upl, lowl = len(ll) // 2, len(ll), 0
        while True:
            lw = list(w)
            for layer in ll[:thr]:
                lw[layer] = b
            a = evaluate(lw)
            evaluations += 1
            met = a >= t
            previous = thr
            if met:      # the target holds: try to quantize more layers
                lowl = thr
                thr = thr + (upl - thr) // 2
            else:        # too many: quantize fewer
                upl = thr
                thr = thr - (thr - lowl) // 2
            if thr == previous:
                break
        if ensure_target and not met:
            thr = lowl
        for layer in ll[:thr]:
            w[layer] = b
        ll = ll[:thr]     # only these are tried at the next, lower width
    return w, evaluations


def greedy(ll: Sequence[int], bs: Sequence[int], t: float, evaluate: Evaluate) -> Tuple[List[int], int]:
    """Alg. 2.  One layer at a time is lowered to b; it keeps b if the model still meets the target,
    otherwise it returns to its last working width and drops out of the later, lower widths."""
    n = len(ll)
    w = [max(bs)] * n
    ll = list(ll)
    evaluations = 0
    for b in bs:
        ql = []
        for layer in ll:
            last_working = w[layer]
            w[layer] = b
            a = evaluate(list(w))
            evaluations += 1
            if a >= t:
                ql.append(layer)
            else:
                w[layer] = last_working
        ll = ql
    return w, evaluations
