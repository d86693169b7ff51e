"""CPU oracle for the Profiler's linear models and the Partitioner (Algorithm 1) of NeuroFlux
(arXiv 2402.14139, "Modules").  TEST INFRASTRUCTURE ONLY: plain Python, the algorithm's steps
in the paper's order and notation.  Shares nothing with the GPU library.

Pins (tests/test_partition.py): the paper's printed per-layer maximum batch sizes (motivation
figure, VGG-19 under 630 MB) with a hand evaluation of Algorithm 1; the closed form "a block
boundary lies exactly between consecutive layers whose batch sizes differ by more than rho times
the first"; numpy.polyfit and the two-point line for the regression on the paper's printed
memory-versus-batch-size series (VGG-11 figure of the Profiler paragraph).
"""
from __future__ import annotations

import math


def fit_linear(batches, mem):
    """Profiler: least-squares line mem ~ intercept + slope * batch through the measured points
    (normal equations written out).  Returns (slope, intercept)."""
    n = len(batches)
    assert n == len(mem) and n >= 2
    sx = sum(float(b) for b in batches)
    sy = sum(float(m) for m in mem)
    sxx = sum(float(b) * float(b) for b in batches)
    sxy = sum(float(b) * float(m) for b, m in zip(batches, mem))
    den = n * sxx - sx * sx
    slope = (n * sxy - sx * sy) / den
    return slope, (sy - slope * sx) / n


def max_batch(model, M):
    """Algorithm 1, first loop: the largest batch size whose predicted memory stays within the
    budget M (0 if not even one sample fits)."""
    slope, intercept = model
    if slope <= 0:
        return 2 ** 31 - 1 if intercept <= M else 0
    return max(0, int(math.floor((M - intercept) / slope + 1e-12)))


def partition(models, M, B, rho):
    """Algorithm 1.  models: per-layer (slope, intercept); M memory budget; B batch size limit;
    rho grouping threshold.  Returns (b, blocks): the per-layer capped batch sizes and the list
    of blocks as (list of 0-based layer indices, batch size)."""
    b = [min(max_batch(R, M), B) for R in models]
    return b, group(b, rho)


def group(b, rho):
    """Algorithm 1, second loop, on given per-layer batch sizes b: walk the layers; a block
    grows while the next layer's batch size differs from the current layer's by at most
    rho * (current layer's); the block takes the smallest batch size of its layers; the outer
    walk resumes after the layers the block consumed."""
    blocks = []
    n = len(b)
    i = 0
    while i < n:
        layers = [i]
        batch = b[i]
        while i + 1 < n and abs(b[i + 1] - b[i]) <= rho * b[i]:
            batch = min(batch, b[i + 1])
            layers.append(i + 1)
            i += 1
        blocks.append((layers, batch))
        i += 1
    return blocks
