"""Seeded synthetic inputs and the named workload shapes.

Shared by the oracle-side tests and the GPU-side tests/benchmark so that both
see bit-identical inputs.  Holds none of the method's arithmetic.
"""
from .configs import CONFIGS, Workload, get  # noqa: F401
from .generator import generate_numpy, generate_torch, half_bits_to_float, to_half_bits  # noqa: F401
from .special16 import SPECIAL, special_payload  # noqa: F401
