"""Seeded synthetic inputs and the shapes of the benchmark configurations.

This package is the only code shared by the CPU oracle's tests and the HIP
path's tests/benchmark.  It contains no arithmetic of the method itself: it
draws random numbers, rounds them to the storage precision and names shapes.
"""
from .inputs import (  # noqa: F401
    round_to_bf16,
    bf16_bits,
    bits_to_f32,
    gemm_inputs,
    layer_inputs,
    LayerShape,
    token_inputs,
)
from .configs import CONFIGS, GemmCase, gemm_cases  # noqa: F401
