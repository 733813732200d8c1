"""Seeded synthetic inputs for the GRACE-MoE layer hot path.

This package only draws random numbers and lays out tables.  It holds none of
the layer's arithmetic (no gating, no replica pick, no permutation, no FFN):
the CPU oracle and the HIP library both consume the arrays produced here and
share nothing else.
"""
from .generator import (  # noqa: F401
    CONFIGS,
    LayerConfig,
    Placement,
    Workload,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_placement,
    make_workload,
)
