#!/usr/bin/env python3
"""Size sweeps in the style of the paper's evaluation figures (section 6.3: square matrix
sizes for the fp32 and the bf16 matrix product, array sizes for the prefix scan), on one
MI355X.  For context each row also times the vendor routine on the same box and the same
data (torch.matmul, which calls the vendor BLAS, and torch.cumsum): the paper compares its
kernels with the vendor libraries of its GPUs in the same way.  The vendor numbers are
context, not a dependency of the library.

Prints a Markdown table; `bench.py` remains the one-line benchmark.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def timed(fn, stream, reps, warmup=3, ramp_seconds=0.15):
    """Microseconds per call from stream events, after enough untimed calls for the clock
    governor to reach its sustained state (the same for both libraries)."""
    import time
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < ramp_seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e3  # microseconds


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=20)
    args = ap.parse_args()
    import torch
    import paper_2511_11939_amd as P

    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device="cuda").manual_seed(0x5EED)
    lines = []

    lines += ["### bf16 matrix product, M = N = K, A row-major, B column-major, bf16 result", "",
              "| size | this library µs | TFLOP/s | vendor BLAS µs (context) | ratio |", "|---|---|---|---|---|"]
    for n in (1024, 2048, 3072, 4096, 5120, 6144, 8192):
        a = torch.randn(n, n, device="cuda", generator=gen).to(torch.bfloat16)
        b = torch.randn(n, n, device="cuda", generator=gen).to(torch.bfloat16)   # stored [N, K]: column-major K x N
        c = torch.empty(n, n, device="cuda", dtype=torch.bfloat16)
        desc = P.make_desc()
        ws = None
        s, nbytes = P.prism_gemm_workspace_size(desc, n, n, n, 1)
        if nbytes:
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            desc.workspace, desc.workspace_bytes = ws.data_ptr(), nbytes
        mine = timed(lambda: P.gemm(a, b, c, M=n, N=n, K=n, desc=desc, stream=stream), stream, args.reps)
        ref = torch.matmul(a, b.t())
        assert torch.allclose(c.float(), ref.float(), rtol=2e-2, atol=2e-2 * float(n) ** 0.5)
        vend = timed(lambda: torch.matmul(a, b.t()), stream, args.reps)
        lines.append(f"| {n} | {mine:.1f} | {2.0 * n ** 3 / mine / 1e6:.0f} | {vend:.1f} | {vend / mine:.2f} |")

    lines += ["", "### fp32 matrix product C <- 1.5 A B + 0.5 C, M = N = K, all row-major", "",
              "| size | this library µs | TFLOP/s | vendor BLAS µs (context) | ratio |", "|---|---|---|---|---|"]
    for n in (1024, 2048, 3072, 4096):
        a = torch.rand(n, n, device="cuda", generator=gen) * 2 - 1
        b = torch.rand(n, n, device="cuda", generator=gen) * 2 - 1
        c0 = torch.randn(n, n, device="cuda", generator=gen)
        c = c0.clone()
        desc = P.make_desc(ab_dtype="f32", c_dtype="f32", layout_b="row", alpha=1.5, beta=0.5)
        _, nbytes = P.prism_gemm_workspace_size(desc, n, n, n, 1)
        if nbytes:
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            desc.workspace, desc.workspace_bytes = ws.data_ptr(), nbytes
        P.gemm(a, b, c, M=n, N=n, K=n, desc=desc, stream=stream)
        ref = torch.addmm(c0.double(), a.double(), b.double(), beta=0.5, alpha=1.5)
        assert torch.allclose(c.double(), ref, rtol=1e-4, atol=1e-3)
        mine = timed(lambda: P.gemm(a, b, c, M=n, N=n, K=n, desc=desc, stream=stream), stream, args.reps)
        out = torch.empty_like(c0)
        vend = timed(lambda: torch.addmm(c0, a, b, beta=0.5, alpha=1.5, out=out), stream, args.reps)
        lines.append(f"| {n} | {mine:.1f} | {2.0 * n ** 3 / mine / 1e6:.1f} | {vend:.1f} | {vend / mine:.2f} |")

    lines += ["", "### inclusive prefix sum, uint32 (vendor context: torch.cumsum on int32, the same bits)", "",
              "| elements | this library µs | GB/s | torch.cumsum µs (context) | ratio |", "|---|---|---|---|---|"]
    for lg in (20, 22, 24, 26, 28, 30):
        n = 1 << lg
        x = torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), device="cuda", dtype=torch.int32, generator=gen)
        out = torch.empty_like(x)
        _, nbytes = P.prism_scan_workspace_size(n)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        mine = timed(lambda: P.scan_u32(x, out, n, ws, stream=stream), stream, args.reps)
        assert P.prism_scan_check(ws, stream.cuda_stream) == 0
        ref = torch.empty_like(x)
        vend = timed(lambda: torch.cumsum(x, 0, dtype=torch.int32, out=ref), stream, max(3, args.reps // 4))
        assert torch.equal(out, ref)
        lines.append(f"| 2^{lg} | {mine:.1f} | {8.0 * n / mine / 1e3:.0f} | {vend:.1f} | {vend / mine:.2f} |")
        del x, out, ref, ws

    print("\n".join(lines))
    return 0


if __name__ == "__main__":
    sys.exit(main())
