"""Seeded synthetic inputs shaped like VGGT global-attention activations.

This package holds input generation only: no pooling, scoring, selection or
attention arithmetic lives here, so both the CPU oracle's tests and the GPU
path's tests can draw the same tensors from it without sharing any of the
method's code.
"""
from .synthetic import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    generate_head,
    generate,
    round_to_bf16_bits,
    bf16_bits_to_f32,
    num_blocks,
)
