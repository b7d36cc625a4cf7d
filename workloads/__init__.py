"""Seeded synthetic MoE-layer workloads shared by the CPU oracle's tests and the HIP path.

This package only produces *inputs* (shapes, bf16 bit patterns, gate biases).  It holds
none of the MoE arithmetic: no router, no permutation, no FFN, no combine.
"""
from .configs import MoEConfig, CONFIGS, get_config, scaled_config  # noqa: F401
from .gen import (  # noqa: F401
    normal_bf16, gate_bias, make_layer_inputs, LayerInputs, bf16_bits_to_f32, f32_to_bf16_bits,
    torch_bf16_to_u16, u16_to_torch_bf16,
)
