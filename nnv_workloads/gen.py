"""Seeded random weights and inputs for a ConvLayer.

Weights are He-normal, N(0, 2/(C/groups * R * S)) (the single-layer workload
uses N(0, 0.1^2)); inputs are U(-1, 1).  Values are drawn in float64 from a
PCG64 stream seeded by (BASE_SEED + 1000 * stack index + layer index), weights
first, then the input, and rounded to float32 once.
"""
from __future__ import annotations

import math

import numpy as np

from .stacks import ConvLayer, STACK_NAMES

BASE_SEED = 220607446


def layer_seed(stack_name: str, layer_idx: int) -> int:
    return BASE_SEED + 1000 * (STACK_NAMES.index(stack_name) + 1) + layer_idx


def layer_tensors(layer: ConvLayer, seed: int, w_std: float | None = None):
    """Return (w, x): float32 OIHW weights (K, C/groups, R, S) and float32 NCHW input."""
    rng = np.random.default_rng(seed)
    if w_std is None:
        w_std = math.sqrt(2.0 / (layer.cg * layer.r * layer.s))
    w = rng.standard_normal((layer.k, layer.cg, layer.r, layer.s)) * w_std
    x = rng.uniform(-1.0, 1.0, (layer.n, layer.c, layer.h, layer.w))
    return w.astype(np.float32), x.astype(np.float32)
