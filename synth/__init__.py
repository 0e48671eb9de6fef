"""Seeded synthetic inputs (tensors and block masks) for block-sparse attention.

This package only draws random numbers and rounds them to bf16; it holds none of the
attention or planning arithmetic.  Both the CPU oracle's tests and the HIP path's tests
and benchmark take their inputs from here, so the two sides see identical bits.
"""

from .tensors import bf16_bits_to_f32, f32_to_bf16_bits, normal_bf16, qkv_for_config  # noqa: F401
from .masks import (  # noqa: F401
    CONFIGS,
    config_shape,
    imbalance_sweep_mask,
    mask_for_config,
    mask_sequence_cfg5,
    random_mask,
    refine_to_half_blocks,
)
