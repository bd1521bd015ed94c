"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds no arithmetic of the method: only a counter-based random
generator, bf16 bit conversion, the tensor recipes of the benchmark
configurations and the SDXL-shaped layer table as plain data.
"""
from .rng import normal, to_bf16_bits, from_bf16_bits, round_bf16  # noqa: F401
from . import configs, unet_table  # noqa: F401
