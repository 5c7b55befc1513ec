"""Seeded synthetic workloads: operator graphs of the model zoo, inputs, raw weights.

This package is the only code shared by the CPU oracle and the GPU library's
tests.  It holds data descriptions and random-number draws only: no operator
arithmetic, no BN folding, no rounding to storage types.
"""
from .graph import OpSpec, ModelSpec, GraphBuilder  # noqa: F401
from . import zoo, configs, weights  # noqa: F401
