"""Seeded synthetic inputs for the compress-as-you-prefill hot path.

This package holds input shapes and random draws only.  None of the method's
arithmetic (attention, scoring, selection, merging) lives here; both the CPU
oracle's tests and the GPU tests feed on the same arrays it produces.
"""
from .configs import Segment, Workload, WORKLOADS, get_workload, chunk_ranges
from .generate import layer_inputs, f32_to_bf16_bits, bf16_bits_to_f32
from .torch_io import bits_to_torch, torch_to_bits

__all__ = [
    "Segment", "Workload", "WORKLOADS", "get_workload", "chunk_ranges",
    "layer_inputs", "f32_to_bf16_bits", "bf16_bits_to_f32", "bits_to_torch", "torch_to_bits",
]
