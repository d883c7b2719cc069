"""Hessian-trace sensitivity (paper Sec. 3.2.3, E_Hessian) for the one case that needs no trained
network: a linear layer Y = X W' under a mean-squared-error loss over its M N outputs.

The loss is quadratic in W with Hessian (2 / (M N)) (I_N (x) X'X), so Hutchinson's estimate
Tr(H) = E_v[v' H v] needs only quadratic forms of X: with P random sign vectors v_p of length K,

    Tr(H) ~= (2 / M) * mean_p ||X v_p||^2        (exact value: (2 / M) ||X||_F^2),

and with respect to the layer input X the same with W in place of X and N in place of M.  Both the
probes (mpq_rademacher, or drawn inside mpq_hutchinson_quad_signs) and the quadratic forms
(mpq_hutchinson_quad) are libmpq calls, and so are the mean and its standard error over the P doubles
read back (mpq_hutchinson_trace, host arithmetic).
"""
from __future__ import annotations

from . import mpq


def trace_linear_mse(x, probes: int = 32, seed: int = 0, stream_id: int = 0, ws: mpq.Workspace = None):
    """Hutchinson estimate of Tr(d^2 L / d W^2) for L = mean((X W' - T)^2), from `probes` random
    sign vectors.  x: device fp32 [M x K] (the layer's input activations; pass the weight matrix
    [N x K] for the trace with respect to the input).  Returns (estimate, standard error)."""
    M, K = x.shape
    if K % 16 == 0 and x.data_ptr() % 16 == 0:   # the probes are drawn inside the kernel
        q = mpq.hutchinson_quad_signs(x, seed, stream_id, probes, ws=ws).cpu().numpy()
    else:
        v = mpq.rademacher(seed, stream_id, probes, K, device=x.device)
        q = mpq.hutchinson_quad(x, v, ws=ws).cpu().numpy()
    est, err = mpq.hutchinson_trace(q, M)   # mean and standard error: host arithmetic in the library
    return est, err


def order_by_trace(tensors, probes: int = 32, seed: int = 0):
    """Tensors (device fp32 2-D) in ascending order of their estimated Hessian trace: the order in
    which Alg. 1 / Alg. 2 would try to lower precisions under this metric (least sensitive first).
    Returns (order, traces); tensor i draws its probes from stream i."""
    traces = [trace_linear_mse(t, probes, seed, i)[0] for i, t in enumerate(tensors)]
    order = sorted(range(len(traces)), key=lambda i: (traces[i], i))
    return order, traces
