"""Seeded synthetic inputs for the Sparsely-Gated MoE layer.

This package only draws inputs (tokens, gate matrices, noise, expert weights,
upstream gradients).  It holds none of the layer's arithmetic: no gating, no
top-k, no FFN, no losses.  Both the CPU oracle's tests and the HIP path's tests
take their inputs from here so that the two sides see identical bits.
"""
from .configs import MoEShape, CONFIGS, scaled_config  # noqa: F401
from .generators import (  # noqa: F401
    normal_f32,
    gate_inputs,
    hier_gate_inputs,
    expert_weights,
    expert_weights_all,
    zipf_gate_bias,
    dropout_keep,
    upstream_grad,
    STREAMS,
)
