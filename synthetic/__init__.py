"""Seeded synthetic inputs and workload shapes.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It holds no arithmetic of the tiling method: only
workload shapes, a counter-based random generator and the one-time rounding of
generated values to bfloat16 storage.
"""
from .gen import normal_f32, to_bf16_bits, bf16_bits_to_f32, bf16_bits_to_f64  # noqa: F401
from .configs import CONFIGS, FcChain, ConvLayer  # noqa: F401
