"""Seeded synthetic workloads for the K-FAC hot path.

This package holds only workload descriptions (layer shapes) and seeded random
input generators.  It contains none of the method's arithmetic and is the only
code shared by the CPU oracle's tests and the HIP path's tests/benchmarks.
"""
from .shapes import Layer, CONFIGS, config_layers, config_hparams  # noqa: F401
from .inputs import layer_inputs, SEED_ROOT  # noqa: F401
