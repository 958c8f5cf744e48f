"""Seeded synthetic inputs (configs, weights, prompts) shared by the CPU oracle's
tests and by the HIP path's tests and benchmark.

This package holds no arithmetic of the draft-verify method: it only names the
model shapes and draws random numbers.  Neither the oracle nor the HIP library
lives here, and neither of them is imported from here.
"""
from .configs import HivisConfig, CONFIGS, get_config
from .inputs import (TENSOR_ORDER_LAYER, make_weights, make_prompt, to_bf16_bits,
                     bf16_bits_to_f32, round_to_bf16, tensor_rng)

__all__ = ["HivisConfig", "CONFIGS", "get_config", "TENSOR_ORDER_LAYER", "make_weights",
           "make_prompt", "to_bf16_bits", "bf16_bits_to_f32", "round_to_bf16", "tensor_rng"]
