"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package holds only data recipes: model shapes, seeded weight tensors,
prompts and corrupted draft windows.  It contains none of the decoder's or the
verify pass's arithmetic, and imports neither the oracle nor the HIP binding.
"""
from .shapes import ModelShape, SHAPES, shape_by_name
from .tensors import (TENSOR_NAMES, LAYER_TENSORS, GLOBAL_TENSORS, tensor_dims,
                      tensor_f32, tensor_bits, round_to_bf16_bits, bf16_bits_to_f32,
                      WeightStore)
from .tokens import prompt_tokens, corrupt_drafts, rollback_points

__all__ = [
    "ModelShape", "SHAPES", "shape_by_name",
    "TENSOR_NAMES", "LAYER_TENSORS", "GLOBAL_TENSORS", "tensor_dims",
    "tensor_f32", "tensor_bits", "round_to_bf16_bits", "bf16_bits_to_f32",
    "WeightStore", "prompt_tokens", "corrupt_drafts", "rollback_points",
]
