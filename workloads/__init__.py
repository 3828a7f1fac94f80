"""Seeded synthetic MTLA workloads shared by the tests, the bench and the CPU oracle.

This package holds input generation only: Gaussian token streams and weights,
and the projections, LayerNorm and rotary embedding that sit *outside* the
library boundary (they prepare what the library receives).  It contains none
of the arithmetic of the attention path itself and imports neither the HIP
binding nor the oracle.
"""
from .synth import (  # noqa: F401
    Workload, WORKLOADS, Weights, Tokens, make_weights, make_tokens,
    prefix_lengths, bf16_round, bf16_bits, bits_to_f32, rope_rotate,
    sinusoidal_pe, layer_norm, storage_round,
)
