"""Seeded synthetic inputs and network shapes for the integer-CNN hot path.

This package holds only what describes a workload: a counter-based random
generator, tensor shapes and network topologies, and stored calibration
integers.  It contains none of the method's arithmetic (no convolution, no
requantisation, no rounding rule), so both the CPU oracle and the HIP path
may draw their inputs from it without sharing any computation.
"""
from .rng import uniform_int, splitmix64  # noqa: F401
