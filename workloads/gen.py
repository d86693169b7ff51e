"""Seeded random inputs (shapes and draws only; none of the method's arithmetic).

The generator is numpy's counter-based Philox stream keyed by (seed, stream id), so any
tensor can be drawn independently of the others and of the order of calls.  Recipe, as the
benchmark configurations state it: inputs i.i.d. N(0,1) float32, labels i.i.d. uniform over
the classes, convolution / projection / linear weights N(0, 2/fan_in) ("Kaiming normal"),
biases zero (or small N(0, 0.1^2) draws when ``bias_std`` is given, for tests that must
exercise the bias terms).
"""
from __future__ import annotations

import zlib

import numpy as np


def rng_for(seed: int, *stream) -> np.random.Generator:
    """Independent generator for (seed, stream...): Philox keyed by a hash of the stream id."""
    key = zlib.crc32(repr(stream).encode())
    return np.random.Generator(np.random.Philox(key=[int(seed) & 0xFFFFFFFFFFFFFFFF, key]))


def gen_batch(seed: int, batch_index: int, B: int, shape, n_classes: int, dtype=np.float32):
    """One batch of raw inputs [B,C,H,W] ~ N(0,1) and labels [B] uniform on [0,n_classes)."""
    g = rng_for(seed, "batch", batch_index)
    x = g.standard_normal((B,) + tuple(shape)).astype(dtype)
    y = g.integers(0, n_classes, size=(B,), dtype=np.int64).astype(np.int32)
    return x, y


def _kaiming(g, shape, fan_in, dtype):
    return (g.standard_normal(shape) * np.sqrt(2.0 / fan_in)).astype(dtype)


def gen_layer_params(seed: int, layer_index: int, spec, n_classes: int, dtype=np.float32,
                     bias_std: float = 0.0, pool_oh: int = 2, pool_ow: int = 2):
    """Parameters of one local layer and its head: dict W,b,Wp,Wa,ba,Wf,bf (Wp None unless
    the layer has a projection shortcut)."""
    g = rng_for(seed, "params", layer_index)
    K, C, R, S, A = spec.C_out, spec.C_in, spec.R, spec.S, spec.A
    F = A * pool_oh * pool_ow

    def bias(n):
        if bias_std:
            return (g.standard_normal((n,)) * bias_std).astype(dtype)
        return np.zeros((n,), dtype)

    p = {"W": _kaiming(g, (K, C, R, S), C * R * S, dtype), "b": bias(K)}
    p["Wp"] = _kaiming(g, (K, spec.skip_C), spec.skip_C, dtype) if spec.skip_kind == 2 else None
    p["Wa"] = _kaiming(g, (A, K, 3, 3), K * 9, dtype)
    p["ba"] = bias(A)
    p["Wf"] = _kaiming(g, (n_classes, F), F, dtype)
    p["bf"] = bias(n_classes)
    return p


def gen_class_patterns(seed: int, N: int, shape, n_classes: int, noise: float = 0.7, dtype=np.float32):
    """A learnable stand-in data set: every class has a fixed N(0,1) pattern; a sample is its
    class's pattern plus ``noise`` * N(0,1).  Returns (x [N,C,H,W], labels [N] int32)."""
    g = rng_for(seed, "class-patterns", n_classes)
    patterns = g.standard_normal((n_classes,) + tuple(shape))
    y = g.integers(0, n_classes, size=(N,), dtype=np.int64).astype(np.int32)
    x = patterns[y] + noise * g.standard_normal((N,) + tuple(shape))
    return x.astype(dtype), y
