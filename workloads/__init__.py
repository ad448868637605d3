"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path's tests.

This package holds model shapes, workload shapes and random input generators only.
It contains none of the decoder's or the sampler's arithmetic, so that the oracle
and the HIP library can both be fed from it without sharing any code of the method.
"""
from .configs import ModelShape, Workload, CONFIGS, get_config, tiny_neox, tiny_llama  # noqa: F401
from .synth import (  # noqa: F401
    Weights,
    make_weights,
    make_prompts,
    make_uniforms,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    parity_subset,
)
