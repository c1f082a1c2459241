"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path's tests.

This package only draws random inputs (activations, weights, bias) and converts
them to the storage dtype.  It holds none of the method's arithmetic.
"""
from .workloads import (  # noqa: F401
    Workload,
    WORKLOADS,
    get_workload,
    make_inputs,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
)
