"""Oracle for the deployment estimates of the paper's experiments section ("Compute Latency
Estimates", Table 1): the latency of a mixed-precision model is the combination of the kernel
latencies of its layers at their precisions, its size the parameters at their bit-widths.
Plain Python.  TEST INFRASTRUCTURE ONLY: nothing on the product path may import this module.

Reading: the paper says the kernel latencies are combined "suitably" and gives no formula; layers of
an inference pass run one after the other, so the combination is their sum.  Relative figures are
taken against the same model with every layer at the baseline precision, as the table's
percentages are (they reproduce from its absolute rows)."""
from __future__ import annotations

from typing import Mapping, Sequence


def model_latency(kernel_latency: Sequence[Mapping[int, float]], bits: Sequence[int]) -> float:
    """kernel_latency[l][b]: measured latency of layer l's kernel at precision b; bits[l]: the
    precision the configuration gives layer l."""
    assert len(kernel_latency) == len(bits)
    total = 0.0
    for table, b in zip(kernel_latency, bits):
        total += table[b]
    return total


def relative_latency(kernel_latency, bits, baseline_bits: int) -> float:
    return model_latency(kernel_latency, bits) / model_latency(kernel_latency, [baseline_bits] * len(bits))


def model_size_bytes(parameters: Sequence[int], bits: Sequence[int]) -> float:
    assert len(parameters) == len(bits)
    return sum(p * b / 8.0 for p, b in zip(parameters, bits))


def relative_size(parameters, bits, baseline_bits: int) -> float:
    return model_size_bytes(parameters, bits) / model_size_bytes(parameters, [baseline_bits] * len(bits))
