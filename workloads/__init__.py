"""Seeded synthetic MTLA workloads shared by the tests, the bench and the CPU oracle.

This package holds input generation only: Gaussian token streams and weights,
and the projections, LayerNorm and rotary embedding that sit *outside* the
library boundary of the path calls (they prepare what mtla_cache_append,
mtla_decode_attn and mtla_prefill_attn receive).  It contains none of the
arithmetic of the attention path itself and imports neither the HIP binding
nor the oracle.  For the whole-layer call, whose inputs are the token stream
and the projection weights themselves, only make_x and make_layer_weights
(random numbers, rounding, transposes) are used: the projections, LayerNorm and
rotary embedding of that call are computed by the library and, independently,
by the oracle.
"""
from .synth import (  # noqa: F401
    Workload, WORKLOADS, Weights, Tokens, make_weights, make_tokens,
    prefix_lengths, bf16_round, bf16_bits, bits_to_f32, rope_rotate,
    sinusoidal_pe, layer_norm, storage_round, LayerWeights, make_layer_weights, make_x,
)
