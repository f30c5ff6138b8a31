"""Seeded synthetic inputs shaped like VGGT-1B activations and weights.

This package holds data generation only: random draws, outlier structure and
dtype packing.  It contains none of the quantized-linear method's arithmetic
and is the only code shared by the CPU oracle's tests and the HIP path's tests.
"""
from .vggt_inputs import (  # noqa: F401
    TOKENS_PER_FRAME,
    SPECIAL_TOKENS,
    LayerSpec,
    layer_spec,
    config_layers,
    make_weights,
    make_bias,
    make_signs,
    make_activation_frames,
    make_activation_rows,
    make_calibration,
    outlier_channels,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
)
