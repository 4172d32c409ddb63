"""Seeded synthetic inputs shared by the oracle-side tests and the HIP-side harness.

This package holds no arithmetic of the method (no quantizer, no codec, no GEMV): only
shapes, seeds, random draws and the bf16 rounding of the activations that both sides receive.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    MatrixSpec,
    config_matrices,
    make_weights,
    make_activations,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    small_case,
)
