"""Seeded synthetic inputs for the routed quantization-expert forward pass.

This package only draws random tensors of the right shape and lists the
workload configurations.  It holds none of the method's arithmetic (no
quantizer, no router, no GEMM): the CPU oracle and the HIP library both
consume what it produces and share nothing else.
"""
from .configs import CONFIGS, ExpertSpec, WorkloadConfig, get_config, scaled
from .generate import (bf16_bits_to_f32, f32_to_bf16_bits, make_activations,
                       make_cv_router, make_fp_weights, make_image_activations, make_nlp_router, make_router, make_targets,
                       make_token_activations)

__all__ = [
    "CONFIGS", "ExpertSpec", "WorkloadConfig", "get_config", "scaled",
    "bf16_bits_to_f32", "f32_to_bf16_bits", "make_activations",
    "make_fp_weights", "make_router", "make_targets", "make_nlp_router", "make_token_activations", "make_cv_router", "make_image_activations",
]
