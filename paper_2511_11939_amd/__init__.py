"""MI355X (gfx950) dense GEMM and prefix-scan library: Python binding of the C ABI in
include/prism_gemm.h and include/prism_scan.h.

Everything numeric runs in the HIP kernels of libprism_gemm.so; this package
only marshals arguments.  There is no CPU fallback: without the built library
every call raises.
"""
from .binding import (  # noqa: F401
    GemmDesc, GemmPlan, PrismError, Status, DType, Layout,
    load_library, library_path,
    prism_gemm, prism_gemm_batched, prism_gemm_workspace_size, prism_gemm_plan,
    prism_gemm_batched_stamped, STAMP_BYTES_PER_WORKGROUP,
    prism_sched_map, prism_status_string, prism_version, prism_mfma_probe, prism_layout_probe, prism_reread_environment,
    LAYOUT_ACCUMULATOR_BF16, LAYOUT_ACCUMULATOR_F16, LAYOUT_K_ROWS_READ,
    MFMA_PROBE_OPERAND_BYTES, MFMA_PROBE_COUNTER_BYTES, MFMA_PROBE_FLOP_PER_ITERATION,
    gemm, make_desc,
    prism_scan_workspace_size, prism_scan_u32, prism_scan_check, prism_scan_u32_static, scan_u32,
)
