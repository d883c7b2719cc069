"""Kernel latency table of mpq_qgemm on this GPU and the mixed-precision latency / footprint
estimate built from it.

The paper estimates the deployment latency of a bit configuration by benchmarking its GEMM / conv
kernels per precision at inference batch size one and combining the kernel latencies of the
layers (experiments section, "Compute Latency Estimates"); the A100 / CUTLASS figures themselves do
not carry over to other hardware, the procedure does.  Here the kernel is mpq_qgemm, the
precisions are the two it has (weights stored as int8 or as packed int4, activations int8), and
the combination is the sum over layers.  Everything on the device runs through libmpq; torch
supplies buffers and the events that time the launches.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Iterable, List, Sequence, Tuple

from . import mpq

Shape = Tuple[int, int, int]          # (M, K, N) of one linear layer, weights [N x K]


def storage_bits(bits: int) -> int:
    """How a weight tensor of width `bits` is stored for the GEMM: packed int4 up to 4 bits."""
    return 4 if bits <= 4 else 8


def time_qgemm(M: int, K: int, N: int, w_storage_bits: int, reps: int = 40, warmup: int = 5,
               cold_bytes: int = 320 << 20) -> float:
    """Average time of one mpq_qgemm launch in microseconds, launches back to back.  Operands
    rotate over enough buffers that no launch finds its inputs in the 256 MB last-level cache
    (at most 64 buffers): a layer's weights are cold when inference reaches it."""
    import torch
    per_launch = M * K + N * K * w_storage_bits // 8 + 4 * M * N
    nbuf = max(2, min(64, -(-cold_bytes // per_launch)))
    dev = "cuda"
    g = torch.Generator(device=dev).manual_seed(1)
    a = [torch.randint(-127, 128, (M, K), dtype=torch.int8, device=dev, generator=g) for _ in range(nbuf)]
    wshape = (N, K) if w_storage_bits == 8 else (N, K // 2)
    wdt = torch.int8 if w_storage_bits == 8 else torch.uint8
    lo, hi = (-127, 128) if w_storage_bits == 8 else (0, 256)
    w = [torch.randint(lo, hi, wshape, dtype=wdt, device=dev, generator=g) for _ in range(nbuf)]
    y = [torch.empty((M, N), dtype=torch.float32, device=dev) for _ in range(nbuf)]
    sa = torch.full((1,), 0.01, dtype=torch.float32, device=dev)
    sw = torch.full((N,), 0.001, dtype=torch.float32, device=dev)
    ws = mpq.Workspace()

    def launch(i):
        mpq.qgemm(a[i % nbuf], w[i % nbuf], sa, sw, w_storage_bits, mpq.PER_ROW, y=y[i % nbuf], ws=ws)

    for i in range(warmup):
        launch(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda._sleep(2_000_000)   # the host queues the launches while the GPU is held
    e0.record()
    for i in range(reps):
        launch(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


@dataclass
class LatencyTable:
    """microseconds per (M, K, N, weight storage bits).

    Precision axes: the paper times a kernel per (shape, precision).  On this hardware and in this
    library the precision of a layer is a pair (weight bits, activation bits), and it maps to a
    kernel as follows: weights of up to 4 bits travel as packed int4 (half the weight bytes, expanded
    to int8 on their way into the matrix core), wider ones as int8; activations are int8 codes at
    every width from 2 to 8 (a 4-bit activation is an int8 code in +-7).  gfx950 has no integer
    matrix instruction narrower than int8, so the activation width selects no other kernel and no
    other amount of traffic: the table is indexed by weight storage only, and lookup() accepts the
    activation width for completeness and ignores it."""
    us: Dict[Tuple[int, int, int, int], float] = field(default_factory=dict)

    def measure(self, shapes: Iterable[Shape], storages: Sequence[int] = (8, 4), **kw) -> "LatencyTable":
        for (M, K, N) in shapes:
            for st in storages:
                if (M, K, N, st) not in self.us and not (st == 4 and K % 2):
                    self.us[(M, K, N, st)] = time_qgemm(M, K, N, st, **kw)
        return self

    def lookup(self, shape: Shape, bits: int, act_bits: int = 8) -> float:
        if not 2 <= act_bits <= 8:
            raise ValueError("activations are int8 codes of 2..8 bits")
        return self.us[(shape[0], shape[1], shape[2], storage_bits(bits))]

    def estimate_us(self, layers: Sequence[Shape], bits: Sequence[int], act_bits: Sequence[int] = None) -> float:
        """Latency estimate of a configuration: the kernel latencies of its layers, added up
        (mpq_latency_estimate on the rows of the table that belong to the layers)."""
        if len(layers) != len(bits) or (act_bits is not None and len(act_bits) != len(bits)):
            raise ValueError("one bit-width per layer")
        act_bits = act_bits or [8] * len(bits)
        for s, b, a in zip(layers, bits, act_bits):
            self.lookup(s, b, a)   # raises KeyError for a shape that was not measured
        storages = (8, 4)
        rows = [[self.us.get((s[0], s[1], s[2], st), float("nan")) for st in storages] for s in layers]
        return mpq.latency_estimate(rows, [storages.index(storage_bits(b)) for b in bits])

    def relative(self, layers: Sequence[Shape], bits: Sequence[int], baseline_bits: int = 8) -> float:
        """Estimated latency relative to every layer at baseline_bits (the paper's relative latency)."""
        return self.estimate_us(layers, bits) / self.estimate_us(layers, [baseline_bits] * len(layers))


def footprint_bytes(layers: Sequence[Shape], bits: Sequence[int]) -> float:
    """Model footprint of a configuration: parameters times their bit-width (mpq_model_size_bytes)."""
    return mpq.model_size_bytes([s[1] * s[2] for s in layers], bits)


def relative_footprint(layers: Sequence[Shape], bits: Sequence[int], baseline_bits: int = 8) -> float:
    return footprint_bytes(layers, bits) / footprint_bytes(layers, [baseline_bits] * len(layers))
