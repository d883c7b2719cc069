"""Seeded synthetic inputs and shape tables for the five benchmark configurations.

This module holds NO arithmetic of the method (no quantizer, no error sum, no RNG of the noise
path): only shapes and numpy random draws.  It is the one module both the HIP path's callers and
the CPU oracle's callers may import, so both sides see identical arrays.

The tensors stand in for the ResNet-50 / ImageNet and BERT / SQuAD workloads of the paper's
experiments section (datasets and trained weights are not available): layer shapes are the real
ones, values are drawn from the distributions listed per configuration below.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Tuple

import numpy as np


@dataclass(frozen=True)
class Gemm:
    """One linear layer: activations A [M x K], weights W [N x K] (out x in, K contiguous)."""
    name: str
    M: int
    K: int
    N: int


# --- configuration 1: one small linear layer -------------------------------------------------
CFG1 = [Gemm("linear", 64, 256, 256)]

# --- configuration 2: ResNet-50 bottleneck convs lowered to GEMM at batch 32, 224x224 ---------
# 3x3 convs of the four stages (K = 9*C_in) and 1x1 convs with K = N, each 1x1 paired with the
# stage whose output width it equals.
CFG2 = [
    Gemm("stage1_3x3", 100352, 576, 64),
    Gemm("stage2_3x3", 25088, 1152, 128),
    Gemm("stage3_3x3", 6272, 2304, 256),
    Gemm("stage4_3x3", 1568, 4608, 512),
    Gemm("stage1_1x1", 100352, 256, 256),
    Gemm("stage2_1x1", 25088, 512, 512),
    Gemm("stage3_1x1", 6272, 1024, 1024),
    Gemm("stage4_1x1", 1568, 2048, 2048),
]

# --- configuration 3: BERT-base encoder linears, seq 384 x batch 32 ---------------------------
CFG3 = [
    Gemm("qkv", 12288, 768, 2304),
    Gemm("attn_out", 12288, 768, 768),
    Gemm("ffn1", 12288, 768, 3072),
    Gemm("ffn2", 12288, 3072, 768),
]

# --- configuration 4: BERT-large-sized weight set (24 layers x 4 linears) ---------------------
CFG4_LAYER = [("qkv", 3072, 1024), ("attn_out", 1024, 1024), ("ffn1", 4096, 1024),
              ("ffn2", 1024, 4096)]  # (name, N rows, K cols), stored [N x K]
CFG4_LAYERS = 24

# --- configuration 5: BERT-large FFN block at M = 16384 ---------------------------------------
CFG5 = [Gemm("ffn1", 16384, 1024, 4096), Gemm("ffn2", 16384, 4096, 1024)]
CFG5_CANDIDATES = 64


def _rng(seed: int, *path: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *path])))


def normal_f32(rng: np.random.Generator, shape, sigma: float = 1.0) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return a


# ----------------------------------------------------------------------------------------------
def cfg1_tensors(seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """X [64x256] ~ N(0,1), W [256x256] ~ N(0, 0.05^2)."""
    rng = _rng(seed, 1)
    g = CFG1[0]
    return normal_f32(rng, (g.M, g.K)), normal_f32(rng, (g.N, g.K), 0.05)


def cfg2_layer(idx: int, seed: int = 1, rows: int | None = None):
    """Layer idx of configuration 2: A = |N(0,1)| (post-ReLU), W He-normal (variance 2/K).

    Returns (A, W, bits_A, bits_W); bits drawn uniformly from {4, 8}.  ``rows`` truncates M (the
    leading rows of the full-size draw are NOT reproduced; a truncated draw is its own tensor).
    """
    g = CFG2[idx]
    rng = _rng(seed, 2, idx)
    m = g.M if rows is None else min(rows, g.M)
    a = np.abs(normal_f32(rng, (m, g.K)))
    w = normal_f32(rng, (g.N, g.K), float(np.sqrt(2.0 / g.K)))
    bits = rng.choice([4, 8], size=2)
    return a, w, int(bits[0]), int(bits[1])


def cfg3_layer(idx: int, seed: int = 2, rows: int | None = None):
    """Layer idx of configuration 3: W ~ N(0, 0.02^2); A ~ N(0,1) with six fixed outlier columns
    in which entries are multiplied by 20 with the probability that makes 0.1 % of all entries
    outliers.  Returns (A, W, bits_A, bits_W)."""
    g = CFG3[idx]
    rng = _rng(seed, 3, idx)
    m = g.M if rows is None else min(rows, g.M)
    a = normal_f32(rng, (m, g.K))
    chans = rng.choice(g.K, size=6, replace=False)
    p = min(1.0, 0.001 * g.K / 6.0)
    mask = rng.random((m, 6)) < p
    sub = a[:, chans]
    sub[mask] *= np.float32(20.0)
    a[:, chans] = sub
    w = normal_f32(rng, (g.N, g.K), 0.02)
    bits = rng.choice([4, 8], size=2)
    return a, w, int(bits[0]), int(bits[1])


def bert_large_weight(rows: int, cols: int, rng: np.random.Generator) -> np.ndarray:
    """N(0, 0.02^2) with 0.05 % of entries replaced by +-10 sigma = +-0.2."""
    w = normal_f32(rng, (rows, cols), 0.02)
    n_out = int(round(0.0005 * rows * cols))
    pos = rng.choice(rows * cols, size=n_out, replace=False)
    sign = rng.integers(0, 2, size=n_out).astype(np.float32) * 2.0 - 1.0
    w.reshape(-1)[pos] = np.float32(0.2) * sign
    return w


def cfg4_tensors(seed: int = 3, layers: int = CFG4_LAYERS) -> Iterator[Tuple[str, np.ndarray]]:
    """Yields the 4*layers weight tensors of configuration 4, one at a time (1.2 GB in total)."""
    for layer in range(layers):
        for t, (name, rows, cols) in enumerate(CFG4_LAYER):
            yield "L%02d.%s" % (layer, name), bert_large_weight(rows, cols, _rng(seed, 4, layer, t))


def cfg5_tensors(seed: int = 4, rows: int | None = None):
    """X [M x 1024] ~ N(0,1); W1 [4096x1024], W2 [1024x4096] as configuration 4."""
    rng = _rng(seed, 5)
    m = CFG5[0].M if rows is None else rows
    x = normal_f32(rng, (m, CFG5[0].K))
    w1 = bert_large_weight(CFG5[0].N, CFG5[0].K, rng)
    w2 = bert_large_weight(CFG5[1].N, CFG5[1].K, rng)
    return x, w1, w2


def cfg5_candidates(seed: int = 4, count: int = CFG5_CANDIDATES) -> List[Tuple[int, int, int, int]]:
    """(b_W1, b_A1, b_W2, b_A2) per candidate: weights from {2,4,8}, activations from {4,8}."""
    rng = _rng(seed, 5, 99)
    bw = rng.choice([2, 4, 8], size=(count, 2))
    ba = rng.choice([4, 8], size=(count, 2))
    return [(int(bw[i, 0]), int(ba[i, 0]), int(bw[i, 1]), int(ba[i, 1])) for i in range(count)]


# --- a stack of linear layers for the configuration searches (Alg. 1 / Alg. 2) ----------------
def search_stack(seed: int = 6, layers: int = 8, width: int = 64, rows: int = 128):
    """X [rows x width] ~ N(0,1) and `layers` square He-normal weights N(0, 2/width).  To give the
    layers different sensitivities, 0.2 % of the entries of layer l are set to +-k_l sigma with a
    seeded per-layer k_l in [3, 12]: the larger the outliers, the coarser the grid left for the
    bulk of the weights at a given width."""
    rng = _rng(seed, 6)
    x = normal_f32(rng, (rows, width))
    sigma = float(np.sqrt(2.0 / width))
    k = 3.0 + 9.0 * rng.random(layers)
    weights = []
    for l in range(layers):
        w = normal_f32(rng, (width, width), sigma)
        n_out = max(1, int(round(0.002 * w.size)))
        pos = rng.choice(w.size, size=n_out, replace=False)
        sign = rng.integers(0, 2, size=n_out).astype(np.float32) * 2.0 - 1.0
        w.reshape(-1)[pos] = np.float32(k[l] * sigma) * sign
        weights.append(w)
    return x, weights
