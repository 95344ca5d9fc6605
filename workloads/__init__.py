"""Seeded synthetic inputs for the prefill-attention + prompt-refinement path.

This module only draws numbers and lays them out; it holds none of the
method's arithmetic (no attention, no softmax, no selection).  Both the CPU
checker and the GPU path receive the arrays produced here.

Shapes follow the paper's evaluation workload (long document prompts of
4k-32k tokens refined at a ratio around 0.25, Section 4.1 "Settings"); the
values are synthetic normal draws rounded to bf16.
"""
from .gen import (
    Workload,
    CONFIG_NAMES,
    make_workload,
    make_custom,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    keep_count,
    C3_LENGTHS,
    c3_lengths_from_recipe,
)

__all__ = [
    "Workload",
    "CONFIG_NAMES",
    "make_workload",
    "make_custom",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "keep_count",
    "C3_LENGTHS",
    "c3_lengths_from_recipe",
]
