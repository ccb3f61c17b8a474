"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU harness.

This module holds no arithmetic of the method itself (no convolution, pooling,
loss or swap logic): it only produces the byte-identical input tensors both
sides consume.  Everything is derived from a counter-based generator
(splitmix64 -> uniform -> Box-Muller), so a tensor is a pure function of
(seed, stream id, element index) and does not depend on any library RNG state.

Layouts follow the rest of the repository: activations NDHWC, 3x3x3 weights
[kd][kh][kw][C_in][C_out], 2x2x2 transposed-conv weights [i][j][k][C_in][C_out],
head weights [C][classes].  bf16 tensors are carried as numpy uint16 bit
patterns.
"""
from .rng import (SEED, uniform, normal, f32_to_bf16_bits, bf16_bits_to_f32,
                  round_to_bf16)
from .tensors import (conv_weights, upconv_weights, head_weights, activations,
                      volume_field, ellipsoid_labels, unet_plan, unet_params, bp_plan, bp_params,
                      inverse_frequency_class_weights)

__all__ = [
    "SEED", "uniform", "normal", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "round_to_bf16", "conv_weights", "upconv_weights", "head_weights",
    "activations", "volume_field", "ellipsoid_labels", "unet_plan",
    "unet_params", "bp_plan", "bp_params", "inverse_frequency_class_weights",
]
