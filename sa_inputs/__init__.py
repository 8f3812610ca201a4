"""Seeded synthetic inputs for the SampleAttention hot path.

This module only *makes inputs*: Gaussian Q/K/V, rotary position embedding,
planted attention sinks (column structure) and planted slash offsets (diagonal
structure), rounded once to bf16.  It holds none of the method's arithmetic
(no softmax, no scores, no selection) and is the one module that both the CPU
oracle's tests and the GPU path's tests/bench may share.
"""
from .generator import (  # noqa: F401
    CONFIGS,
    HEAD_PATTERNS,
    Workload,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_group,
    make_inputs,
    rows_from_ratio,
)
