"""Seeded synthetic inputs (model shapes, weights, prompts).

This package is the only code shared by the CPU oracle and the HIP path.  It
holds no arithmetic of the decoding method itself: only the table of model
shapes and a counter-based, integer-only generator for weights and prompts, so
that any element of any tensor can be produced on the CPU or on the GPU with
identical bits.
"""
from .configs import ModelConfig, CONFIGS, get_config
from .generator import (gen_tensor, gen_prompt, gen_uniforms, tensor_shape, iter_tensor_specs,
                        KINDS, GLOBAL_KINDS, LAYER_KINDS)

__all__ = ["ModelConfig", "CONFIGS", "get_config", "gen_tensor", "gen_prompt", "gen_uniforms",
           "tensor_shape", "iter_tensor_specs", "KINDS", "GLOBAL_KINDS", "LAYER_KINDS"]
