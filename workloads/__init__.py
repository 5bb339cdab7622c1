"""Seeded synthetic inputs and layer-shape tables.

This package holds no K-FAC arithmetic.  It only describes layer shapes
(``shapes``) and draws the random tensors (``rng``) that both the CPU oracle
and the HIP library consume, so the two sides see identical bits.
"""
from .shapes import LayerSpec, CONFIGS, config_layers, config_hparams  # noqa: F401
from .rng import draw_normal, draw_relu_normal, to_bf16_bits, bf16_bits_to_f32, layer_inputs  # noqa: F401
