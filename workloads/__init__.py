"""Seeded synthetic inputs for the GEMM and prefix-scan workloads.

This package only draws numbers and rounds them once to their storage type; it
holds none of the arithmetic under test.  Both the CPU oracle's tests and the GPU library's
tests and benchmark take their inputs from here, so that the two sides always
see the same bit patterns.
"""
from .generators import (  # noqa: F401
    uniform_pm1, normal, small_integers, to_bf16_bits, to_f16_bits, encode, scan_input_u32,
)
from .configs import CONFIGS, GemmWorkload, make_inputs  # noqa: F401
