"""Seeded synthetic inputs and the named workload shapes.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds no arithmetic of the training step itself: only shapes,
a counter-based random stream, and the one-time rounding of inputs to the
storage precision, so that both sides start from identical numbers.

The paper trains decoder-only Transformers at sequence length 2048 with heads
split over the tensor-parallel mesh axis (Fig. 1, Sec. 3.2, Table 1 caption)
and names no dataset, so every input here is drawn from a Philox stream:
activations and upstream gradients N(0,1), weight matrices N(0,sigma), biases
0, LayerNorm gain 1 / shift 0, token ids uniform over the vocabulary.
"""
from .configs import CONFIGS, BlockShape, ModelShape, get_config
from .generate import (
    PARAM_NAMES, MATRIX_NAMES, round_to_bf16, bf16_bits, from_bf16_bits,
    make_block_params, make_block_inputs, make_stack_inputs, make_model_inputs,
)

__all__ = [
    "CONFIGS", "BlockShape", "ModelShape", "get_config",
    "PARAM_NAMES", "MATRIX_NAMES", "round_to_bf16", "bf16_bits", "from_bf16_bits",
    "make_block_params", "make_block_inputs", "make_stack_inputs", "make_model_inputs",
]
