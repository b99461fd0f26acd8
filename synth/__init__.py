"""Seeded synthetic inputs for the sparse-FC training step.

This package only draws numbers and lays out shapes: it holds none of the
method's arithmetic and is the one module that both the CPU oracle's tests and
the HIP path's tests / benchmark read their inputs from.
"""
from .inputs import (  # noqa: F401
    LAYER_SETS,
    CONFIGS,
    normal,
    uniform_mask,
    nested_uniform_masks,
    powerlaw_mask,
    to_bf16_bits,
    bf16_bits_to_f32,
    make_layer,
    make_activations,
)
