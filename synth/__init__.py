"""Seeded synthetic-input generators shared by the CPU oracle's tests and the HIP path's tests.

This package holds none of the method's arithmetic: it only produces model weights, prompts, skip
masks and uniform streams as pure functions of (seed, tensor id, index), so that the CPU oracle and
the GPU library can be fed bit-identical inputs without either importing the other.
"""
from .gen import (  # noqa: F401
    CONFIGS, ModelShape, tensor_shapes, tensor_id, gen_tensor_f32, gen_tensor, gen_gain, f32_to_bf16_bits,
    bf16_bits_to_f32, gen_prompt, SEED_WEIGHTS, SEED_MASK, SEED_PROMPT, SEED_UNIFORMS, scale_f32,
    LAYER_SLOTS, GLOBAL_SLOTS, gen_uniforms, gen_skip_mask, gen_sublayer_mask, mix64, HostWeights, gen_host_weights,
)
