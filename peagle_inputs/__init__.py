"""Seeded synthetic inputs shared by the fp64 oracle and the HIP path.

This module holds no attention arithmetic: it names the workload shapes, draws the
random tensors and rounds them to bf16 bit patterns.  Both sides consume exactly
these bytes.
"""
from .gen import (CONFIGS, PAGE_TOKENS, WorkloadConfig, bf16_bits_to_f64, cod_depth_counts, f32_to_bf16_bits,
                  make_decode_inputs, make_inputs, make_inputs_tokens, useful_flops, useful_pairs, useful_pairs_sampled)

__all__ = [
    "CONFIGS",
    "WorkloadConfig",
    "bf16_bits_to_f64",
    "f32_to_bf16_bits",
    "make_inputs",
    "make_inputs_tokens",
    "make_decode_inputs",
    "PAGE_TOKENS",
    "cod_depth_counts",
    "useful_pairs_sampled",
    "useful_pairs",
    "useful_flops",
]
