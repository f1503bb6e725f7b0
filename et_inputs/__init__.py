"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only draws random numbers and shapes them (weights, video clips,
hidden-state tensors).  It holds none of the encoder's or the compression
method's arithmetic, so that the oracle and the HIP path stay independent.
"""
from .bf16 import round_to_bf16, f32_to_bf16_bits, bf16_bits_to_f32
from .shapes import EncoderShape, TINY, SIGLIP
from .weights import make_weights
from .clips import (
    make_clip,
    scene_lengths_fixed,
    scene_lengths_uniform,
    scene_lengths_geometric,
    make_hidden_states,
)
from .workloads import WORKLOADS, build_workload

__all__ = [
    "round_to_bf16", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "EncoderShape", "TINY", "SIGLIP", "make_weights",
    "make_clip", "scene_lengths_fixed", "scene_lengths_uniform",
    "scene_lengths_geometric", "make_hidden_states",
    "WORKLOADS", "build_workload",
]
