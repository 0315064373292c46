"""Seeded synthetic workloads for the VideoScan streaming-attention path.

This package only draws random tensors and names shapes; it contains none of the
method's arithmetic (no attention, no pooling, no cache logic).  Both the GPU
tests/benchmark and the CPU oracle's callers take their inputs from here so that
the two sides see the same bytes.
"""
from .configs import CONFIGS, AttnShape  # noqa: F401
from .gen import (  # noqa: F401
    draw,
    frame_inputs,
    cache_rows,
    carrier_embeddings,
    decode_step_inputs,
    decode_lengths,
    cfg1_inputs,
    to_f64,
    hidden_rows,
    layer_weights,
)
