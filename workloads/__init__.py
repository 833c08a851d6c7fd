"""Seeded synthetic inputs for the STA + GSTA forward path.

This package only *generates inputs* (random embeddings, valid lengths, layer
weights) and converts number formats. It contains none of the method's
arithmetic (no scores, gates, segment sums or attention), so both the CPU
checker and the GPU path may consume what it produces.
"""
from .bf16 import f32_to_bf16_bits, bf16_bits_to_f32, round_to_bf16
from .configs import CONFIGS, WorkloadSpec, Workload, make_workload, make_user

__all__ = [
    "f32_to_bf16_bits", "bf16_bits_to_f32", "round_to_bf16",
    "CONFIGS", "WorkloadSpec", "Workload", "make_workload", "make_user",
]
