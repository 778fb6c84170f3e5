"""Seeded synthetic inputs with the value distributions of the benchmark workloads.

Activations a = max(0, N(0,1)) (or N(0,1) for the transformer workload), output
gradients g ~ N(0, 1e-3^2), weight gradients ~ N(0, 1e-2^2), all drawn in fp32 on
the host.  Each tensor has its own stream keyed by (config, step, layer, kind) so
any single tensor can be regenerated without the others.
"""
from __future__ import annotations

import numpy as np

from .shapes import Layer

SEED_ROOT = 210706533
KIND_ACT, KIND_GOUT, KIND_GRADW = 0, 1, 2


def _rng(cid: int, step: int, layer_idx: int, kind: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED_ROOT, cid, step, layer_idx, kind])))


def activations(layer: Layer, cid: int, step: int, layer_idx: int, relu: bool = True) -> np.ndarray:
    a = _rng(cid, step, layer_idx, KIND_ACT).standard_normal(layer.act_shape, dtype=np.float32)
    if relu:
        np.maximum(a, 0.0, out=a)
    return a


def out_grads(layer: Layer, cid: int, step: int, layer_idx: int, sigma: float = 1e-3) -> np.ndarray:
    g = _rng(cid, step, layer_idx, KIND_GOUT).standard_normal(layer.gout_shape, dtype=np.float32)
    g *= np.float32(sigma)
    return g


def weight_grads(layer: Layer, cid: int, step: int, layer_idx: int, sigma: float = 1e-2) -> np.ndarray:
    v = _rng(cid, step, layer_idx, KIND_GRADW).standard_normal((layer.dG, layer.dA), dtype=np.float32)
    v *= np.float32(sigma)
    return v


def layer_inputs(layer: Layer, cid: int, step: int, layer_idx: int, relu: bool = True):
    """(act, gout, gradW) for one layer of one step, fp32, C-contiguous."""
    return (activations(layer, cid, step, layer_idx, relu),
            out_grads(layer, cid, step, layer_idx),
            weight_grads(layer, cid, step, layer_idx))
