"""The method end to end on a synthetic model, through libmpq only:

    python -m paper_2302_01382_amd.demo [--layers 12] [--width 512] [--rows 2048] [--target 0.9]

1. a stack of linear layers with ReLU between them (seeded weights with layer-dependent outliers),
2. the three sensitivity metrics of Sec. 3.2 per layer -- E_QE (Eq. 2), E_N (Eq. 3-5), the Hessian
   trace of Sec. 3.2.3 for a linear layer under a mean-squared-error loss -- and the order each of
   them puts the layers in,
3. the two searches (Alg. 1 bisection, Alg. 2 greedy) for the lowest-precision configuration whose
   score stays above the target (a fraction of the score with every layer at the widest width),
4. the deployment estimates of the result: model size and latency relative to the widest width
   (kernel latencies measured on this GPU).

The score is 1 - ||Y - Y_ref||^2 / ||Y_ref||^2 against the fp32 output of the unquantized stack: a
stand-in for the task accuracy of the paper, whose datasets and trained weights are not needed here.
"""
from __future__ import annotations

import argparse

from . import hessian, latency, mpq, workloads
from .stack import QuantStack


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--layers", type=int, default=12)
    ap.add_argument("--width", type=int, default=512)
    ap.add_argument("--rows", type=int, default=2048)
    ap.add_argument("--target", type=float, default=0.9, help="score to keep, as a fraction of the all-widest score")
    ap.add_argument("--bits", type=int, nargs="+", default=[8, 4, 2])
    ap.add_argument("--seed", type=int, default=6)
    args = ap.parse_args()

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("the demo needs a GPU: every step runs in libmpq's kernels")
    mpq.lib()
    x, ws = workloads.search_stack(args.seed, args.layers, args.width, args.rows)
    x = torch.from_numpy(x).cuda()
    ws = [torch.from_numpy(w).cuda() for w in ws]
    model = QuantStack(x, ws, args.bits)
    top, low = max(args.bits), sorted(args.bits)[len(args.bits) // 2]
    base = model.evaluate([top] * len(model))
    print("stack: %d layers of %d x %d, %d rows; score with every layer at %d bits: %.6f"
          % (len(model), args.width, args.width, args.rows, top, base))

    # sensitivities at the middle width of the list
    e_qe = model.qe_sensitivity(low)
    e_n = model.noise_sensitivity(low, seed=args.seed)
    # inputs of the layers (fp32 forward pass of the unquantized stack) for the Hessian traces
    inputs, h = [], x
    for i, w in enumerate(ws):
        inputs.append(h.contiguous())
        h = torch.relu(h @ w.t()) if i + 1 < len(ws) else h @ w.t()
    tr = [hessian.trace_linear_mse(a, probes=32, seed=args.seed, stream_id=i)[0] for i, a in enumerate(inputs)]
    print("\nlayer   E_QE(%d bits)   E_N(%d bits)   Hessian trace" % (low, low))
    for l in range(len(model)):
        print("%5d   %12.5f   %11.3e   %13.4e" % (l, e_qe[l], e_n[l], tr[l]))
    orders = {"E_QE": model.order_by(e_qe), "E_N": model.order_by(e_n), "Hessian": model.order_by(tr)}
    for name, order in orders.items():
        print("order by %-8s (least sensitive first): %s" % (name, " ".join(str(l) for l in order)))

    # searches, with the kernel latencies of this GPU for the deployment estimates
    target = args.target * base
    shapes = [(args.rows, w.shape[1], w.shape[0]) for w in ws]
    table = latency.LatencyTable().measure(set(shapes), reps=20, warmup=3)
    print("\ntarget score %.6f (%.4f of the all-%d-bit score)" % (target, args.target, top))
    print("%-8s %-10s %-40s %8s %6s %9s %9s" % ("metric", "search", "bits per layer", "score", "evals", "rel.size", "rel.lat."))
    for name, order in orders.items():
        for search, run in (("bisection", model.bisection), ("greedy", model.greedy)):
            before = model.evaluations
            bits, asked = run(order, target)
            score = model.evaluate_once(bits)
            print("%-8s %-10s %-40s %8.6f %6d %9.3f %9.3f"
                  % (name, search, " ".join(str(b) for b in bits), score, model.evaluations - before,
                     latency.relative_footprint(shapes, bits, top), table.relative(shapes, bits, top)))
    print("\n(evals: evaluations that ran on the GPU; configurations already scored are answered from a table)")


if __name__ == "__main__":
    main()
