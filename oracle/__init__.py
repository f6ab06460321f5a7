"""CPU oracles (GEMM, prefix scan) -- TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this.  Callers allowed: the tests, the
smoke check and the benchmark's CPU-baseline leg.
"""
from .reference import (  # noqa: F401
    build_oracle, gemm_ref, gemm_ref_workload, decode_bits, oracle_threads, inclusive_scan_u32_ref,
)
from .check import (  # noqa: F401
    rne_to_format, acceptance_bound, check_against_oracle, decode_output,
)
