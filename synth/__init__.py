"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

This package draws random tensors and plants structure in them.  It holds none of
the eviction method's arithmetic (no softmax, statistics, allocation, selection).
"""
from .generate import CakeConfig, CONFIGS, make_layer, make_config_inputs  # noqa: F401
