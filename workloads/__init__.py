"""Seeded synthetic inputs for the KV-cache merge step.

This package only draws random tensors of the shapes and distributions the
benchmark configurations name (AR(1) Keys, Gaussian / Student-t Values,
Gaussian Queries, ragged lengths).  It holds none of the merge method's
arithmetic, so both the CPU oracle's tests and the GPU path's tests and
benchmark may feed from it without sharing any computation.
"""

from .configs import WORKLOADS, Workload, get_workload
from .generator import (
    UnitInputs,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    gaussian_unit,
    generate_unit,
    unit_budget,
    unit_lengths,
)

__all__ = [
    "WORKLOADS",
    "Workload",
    "get_workload",
    "UnitInputs",
    "generate_unit",
    "gaussian_unit",
    "unit_lengths",
    "unit_budget",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
]
