"""Seeded synthetic inputs for the GEMM workloads.

This package only draws numbers and rounds them once to 16-bit storage; it
holds no matrix arithmetic.  Both the CPU oracle's tests and the GPU library's
tests and benchmark take their inputs from here, so that the two sides always
see the same bit patterns.
"""
from .generators import (  # noqa: F401
    uniform_pm1, normal, small_integers, to_bf16_bits, to_f16_bits, encode,
)
from .configs import CONFIGS, GemmWorkload, make_inputs  # noqa: F401
