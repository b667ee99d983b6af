"""Seeded synthetic chain workloads.

This package only draws random stage costs and sizes.  It holds none of the
checkpoint solver's arithmetic and is the one module that the CPU oracle's
tests and the GPU path's tests/benchmarks both import.
"""
from .chains import CONFIGS, ChainBatch, make_config, random_chain_batch  # noqa: F401
