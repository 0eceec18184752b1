"""Seeded synthetic inputs for the stage executor and for its CPU oracle.

This module only draws random numbers and stores them in the byte formats the
boundary accepts (fp32, or bf16 bit patterns held in uint16).  It contains none
of the arithmetic of the decoder layer itself: no norm, no rotation, no matmul,
no packing offsets.  Both the HIP path's tests and the oracle's tests take
their inputs from here, so both see exactly the same bytes.
"""
from .gen import (  # noqa: F401
    StageShape,
    CONFIGS,
    bf16_bits_from_f32,
    layer_tensors,
    embed_tensors,
    head_tensors,
    token_ids,
    hidden_states,
    ragged_lengths,
    TENSOR_ORDER_LAYER,
    TENSOR_ORDER_HEAD,
)
