"""Seeded synthetic inputs for the fused linear-cross-entropy path.

This package only draws random numbers and rounds them to the storage type.
It contains none of the method's arithmetic (no logits, no softmax, no
gradients), so both the CPU oracle's tests and the HIP path's tests can feed
from it without sharing any code of the method itself.
"""
from .configs import CONFIGS, Workload, make, bf16_bits_to_f64, f32_to_bf16_bits  # noqa: F401
