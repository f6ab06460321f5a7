#!/usr/bin/env python3
"""Throughput of the GEMM hot path (and of the sgemm and scan workloads) on one MI355X.

A step is one call of prism_gemm(_batched) (or prism_scan_u32) on the named synthetic
workload with the operands already resident in HBM.  Order of a run: the paper's own short
protocol first (5 warm-up + 10 timed launches on a GPU that has seen no load yet: "cold"); for
a workload bound by the matrix pipe, the matrix instructions alone under the same protocol
("mfma_probe": the ceiling and the clock they sustain on this machine); then untimed launches of
the step for --ramp-seconds (the GPU's clock governor needs about 0.1 s of load to reach the
clock it sustains; "clock_ramp"), --warmup untimed steps, and exactly --steps timed steps
between two events on the launch stream.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2516.6      # dense bf16 / fp16 matrix peak of MI355X (256 CU x 4096 FLOP/clk x 2.4 GHz)
PEAK_MFMA_F32_TFLOPS = 157.3   # fp32 matrix peak (256 CU x 256 FLOP/clk x 2.4 GHz)
PEAK_HBM_GBS = 8000.0
ESIZE = {"bf16": 2, "f16": 2, "f32": 4}


def algorithmic_bytes(w) -> float:
    """Each operand read once, the result written once (plus the bias vector)."""
    es = ESIZE[w.ab_dtype]
    c_bytes = w.M * w.N * ESIZE[w.c_dtype] * (2 if w.beta != 0.0 else 1)   # C is also read when beta != 0
    return w.batch * (w.M * w.K * es + w.K * w.N * es + c_bytes) + (w.N * 4 if w.bias else 0)


def source_digest() -> str:
    """Digest of the kernel sources: measured HBM traffic is only reported for the
    sources it was measured on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    files = [f for f in glob.glob(os.path.join(ROOT, "paper_2511_11939_amd", "csrc", "*"))
             if f.endswith((".hip", ".hpp"))]          # sources only: objects differ from build to build
    for f in sorted(files):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (two runs), each divided by the factor the same counter shows on a copy of known size
# (--calibrate-copy).  Summaries under profiles/.  workload -> (bytes, digest of the sources).
MEASURED_TRAFFIC: dict = {
    "cfg2_4096_bf16": (235343597, "8635ac6915c82671"),
    "cfg3_proj_bias": (940361503, "8635ac6915c82671"),
    "cfg4_splitk_f16": (273008576, "8635ac6915c82671"),   # main kernel + reduction
    "cfg5_batched_512": (403201246, "8635ac6915c82671"),
    "scan_u32_2p28": (2157273466, "8635ac6915c82671"),
}


def clock_ramp(step, seconds: float) -> int:
    """Untimed launches of the benchmark's own step for `seconds`: the GPU's clock governor takes
    about a tenth of a second of load to reach the clock it then sustains (measured: 4096^3 bf16
    runs at 107-109 us per launch in the first 10 ms of load and at 92 us from 0.1 s on), and a
    benchmark of 110 launches would otherwise time the ramp, not the kernel.  Returns the number of
    launches made."""
    import torch
    n = 0
    if seconds <= 0:
        return n
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(50):
            step()
        torch.cuda.synchronize()
        n += 50
    return n


def mfma_probe(ab_dtype: str, iterations: int, ramp_seconds: float, launches: int = 20):
    """The matrix instructions alone (prism_mfma_probe: the GEMM's wave tile on register-resident
    N(0,1) operands, `iterations` K steps per launch) under the same protocol as the GEMM: what they
    sustain on this machine right now, and at which shader clock.  Returns the figures and the launch
    (for a later reading of the package power)."""
    import numpy as np
    import torch
    import paper_2511_11939_amd as P
    g = torch.Generator(device="cuda")
    g.manual_seed(0x5EED00AA)
    n = P.MFMA_PROBE_OPERAND_BYTES // (4 if ab_dtype == "f32" else 2)
    vals = torch.randn(n, device="cuda", generator=g)
    ops = vals if ab_dtype == "f32" else vals.to(torch.bfloat16 if ab_dtype == "bf16" else torch.float16)
    counters = torch.zeros(P.MFMA_PROBE_COUNTER_BYTES // 8, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream()
    code = {"bf16": P.DType.BF16, "f16": P.DType.F16, "f32": P.DType.F32}[ab_dtype]

    def step():
        s = P.prism_mfma_probe(code, ops, P.MFMA_PROBE_OPERAND_BYTES, iterations, counters,
                               P.MFMA_PROBE_COUNTER_BYTES, stream.cuda_stream)
        assert s == 0, s

    clock_ramp(step, ramp_seconds)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(launches):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    launch_s = e0.elapsed_time(e1) * 1e-3 / launches
    c = counters.cpu().numpy().reshape(-1, 4)
    cycles, ticks = float(c[:, 0].mean()), float(c[:, 1].mean())
    flop = P.MFMA_PROBE_FLOP_PER_ITERATION * iterations * (0.5 if ab_dtype == "f32" else 1.0)
    loop_s = ticks / 100e6
    out = {"tflops_loop": round(flop / loop_s / 1e12, 1), "tflops_launch": round(flop / launch_s / 1e12, 1),
           "clock_mhz": round(cycles / ticks * 100.0, 0), "cycles_per_k_step": round(cycles / iterations, 1),
           "iterations": iterations, "launch_us": round(launch_s * 1e6, 2),
           "what": "matrix instructions only, N(0,1) operands in registers, 256 workgroups x 4 waves, "
                   "after the same clock ramp; tflops_loop is inside the kernel's loop, tflops_launch per launch"}
    return out, step


def socket_power(step, seconds: float):
    """Package power and per-die shader clocks as the system management tool reports them while
    `step` is launched back to back for `seconds` (after the timed region, so the polling cannot
    disturb it).  The tool runs as a child process; without it, or if it reports nothing, None."""
    import re
    import shutil
    import statistics
    import subprocess
    import threading
    import torch
    tool = shutil.which("amd-smi")
    if tool is None:
        return None
    reports, stop = [], threading.Event()

    def poll():
        while not stop.is_set():
            try:
                reports.append(subprocess.run([tool, "metric", "--power", "--clock"], capture_output=True,
                                              text=True, timeout=10).stdout)
            except Exception:
                return

    poller = threading.Thread(target=poll, daemon=True)
    t0 = time.perf_counter()
    poller.start()
    launches = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(100):
            step()
        torch.cuda.synchronize()
        launches += 100
    stop.set()
    poller.join(timeout=15)
    late = reports[len(reports) // 2:]          # the tool's power figure is an average over about a second
    watts = [float(x) for r in late for x in re.findall(r"SOCKET_POWER:\s*([0-9.]+)\s*W", r)]
    if not watts:
        return None
    clocks = [int(x) for x in re.findall(r"GFX_\d+:\s*\n\s*CLK:\s*(\d+)\s*MHz", late[-1])]
    cap = None
    try:
        smi = shutil.which("rocm-smi")
        if smi:
            out = subprocess.run([smi, "--showmaxpower"], capture_output=True, text=True, timeout=10).stdout
            m = re.search(r"Max Graphics Package Power \(W\):\s*([0-9.]+)", out)
            cap = float(m.group(1)) if m else None
    except Exception:
        cap = None
    return {"socket_power_w": round(statistics.median(watts), 0), "power_cap_w": cap,
            "gfx_clock_mhz_per_die": clocks, "seconds": seconds, "launches": launches, "samples": len(watts),
            "what": "amd-smi metric --power --clock polled while the step runs back to back after the timed region; "
                    "the cap is rocm-smi --showmaxpower"}


def copy_ceiling_gbs(n_bytes: int = 1 << 28, reps: int = 20) -> float:
    """What a plain device copy reaches on this machine right now (bytes read + bytes written per
    second): context for the HBM-bound workloads, measured with events on torch's stream."""
    import torch
    src = torch.ones(n_bytes // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n_bytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def calibrate_copy(n_bytes: int, reps: int) -> int:
    """A plain device copy of known size, for scaling the FETCH_SIZE / WRITE_SIZE counters."""
    import torch
    torch.cuda.set_device(0)
    src = torch.ones(n_bytes // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy_bytes_read": n_bytes, "bytes_written": n_bytes, "reps": reps}))
    return 0


def bench_scan(args) -> int:
    """The prefix-scan workload: n uint32 values far beyond the caches, out of place."""
    import numpy as np
    import torch
    import paper_2511_11939_amd as P
    from workloads import scan_input_u32

    n = 1 << 28
    torch.cuda.set_device(0)
    x = scan_input_u32(0x5EED0007, n)
    d_in = torch.from_numpy(x.view(np.int32)).cuda()
    d_out = torch.empty_like(d_in)
    s, ws_bytes = P.prism_scan_workspace_size(n)
    assert s == 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        P.scan_u32(d_in, d_out, n, ws, stream=stream)

    ramp_launches = clock_ramp(step, args.ramp_seconds)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert P.prism_scan_check(ws, stream.cuda_stream) == 0
    launch_ms = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = wall * 1e3 / args.steps
    nbytes = 8.0 * n                                  # every element read once and written once
    gbs = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (launch_ms * 1e-3) / 1e9
    out = {
        "metric": "uint32 inclusive prefix scan GB/s (8 bytes per element) and % of MI355X HBM peak (1 GPU)",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "scan_u32_2p28", "n": n, "tile": 16384, "workgroups": (n + 16383) // 16384},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None, "kernel": "scan_lookback",
                     "launch_us": round(launch_ms * 1e3, 2)},
        "clock_ramp": {"seconds": args.ramp_seconds, "launches": ramp_launches},
    }
    measured = MEASURED_TRAFFIC.get("scan_u32_2p28")
    if measured and measured[1] == source_digest():
        out["roofline"]["traffic"] = measured[0]
    out["roofline"]["device_copy_gbs"] = round(copy_ceiling_gbs(), 1)
    if not args.no_cpu_baseline:
        from oracle import inclusive_scan_u32_ref
        t0 = time.perf_counter()
        ref = inclusive_scan_u32_ref(x)
        cpu_s = time.perf_counter() - t0
        got = d_out.cpu().numpy().view(np.uint32)
        out["cpu_baseline"] = {"value": round(nbytes / cpu_s / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"all {n} elements, {cpu_s:.2f} s wall"}
        out["parity_on_sample"] = {"ok": bool((got == ref).all()), "mismatches": int((got != ref).sum())}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_4096_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=16384, help="output rows the CPU oracle is timed on")
    ap.add_argument("--ramp-seconds", type=float, default=0.3,
                    help="untimed launches of the same step before the warm-up steps, long enough for the "
                         "GPU's clock governor to reach its sustained state (0 = none)")
    ap.add_argument("--no-power", dest="power", action="store_false",
                    help="skip the package-power reading (a few seconds of extra launches with the management tool polled)")
    ap.add_argument("--no-mfma-probe", dest="mfma_probe", action="store_false",
                    help="skip the matrix-instructions-only probe that is reported beside MFMA-bound workloads")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="BYTES",
                    help="run only a device copy of BYTES (counter calibration under rocprofv3)")
    args = ap.parse_args()
    if args.calibrate_copy:
        return calibrate_copy(args.calibrate_copy, args.steps)
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; --gpus must be 1 "
              "(there is no multi-GPU path to measure)", file=sys.stderr)
        return 2
    if args.workload == "scan_u32_2p28":
        return bench_scan(args)

    import numpy as np
    import torch
    import paper_2511_11939_amd as P
    from workloads import CONFIGS, make_inputs

    w = CONFIGS[args.workload]
    torch.cuda.set_device(0)
    inp = make_inputs(w)
    A = torch.from_numpy(inp["A"] if w.ab_dtype == "f32" else inp["A"].view(np.int16)).cuda()
    B = torch.from_numpy(inp["B"] if w.ab_dtype == "f32" else inp["B"].view(np.int16)).cuda()
    bias = None if inp["bias"] is None else torch.from_numpy(inp["bias"]).cuda()
    C = torch.empty(w.batch * w.M * w.N, dtype=torch.float32 if w.c_dtype == "f32" else torch.int16,
                    device="cuda")
    C_in = None
    if w.beta != 0.0:   # C <- alpha*A*B + beta*C is applied to the same C over and over; |beta| < 1 keeps it bounded
        C_in = torch.from_numpy(inp["C_in"].ravel()).cuda()
        C.copy_(C_in)
    desc = P.make_desc(ab_dtype=w.ab_dtype, c_dtype=w.c_dtype, layout_a=w.layout_a, layout_b=w.layout_b,
                       alpha=w.alpha, beta=w.beta, bias=bias, split_k=w.split_k)
    s, ws_bytes = P.prism_gemm_workspace_size(desc, w.M, w.N, w.K, w.batch)
    assert s == 0
    ws = None
    if ws_bytes:
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        desc.workspace, desc.workspace_bytes = ws.data_ptr(), ws_bytes
    s, plan = P.prism_gemm_plan(desc, w.M, w.N, w.K, A, w.lda(), w.M * w.K, B, w.ldb(), w.K * w.N,
                                C, w.N, w.M * w.N, w.batch)
    assert s == 0

    stream = torch.cuda.current_stream()

    # one step = one call of the C entry point through the binding of the same name; the
    # arguments are prepared once, so that the host adds as little as possible to the timed region
    call = (desc, w.M, w.N, w.K, A.data_ptr(), w.lda(), w.M * w.K, B.data_ptr(), w.ldb(), w.K * w.N,
            C.data_ptr(), w.N, w.M * w.N, w.batch, stream.cuda_stream)

    def step():
        status = P.prism_gemm_batched(*call)
        if status != 0:
            raise P.PrismError(status, "prism_gemm_batched")

    def timed(warmup: int, steps: int):
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(steps):
            step()
        ev1.record(stream)
        # (called while the last steps still run, the synchronisation's own round trip to the GPU is hidden
        # behind them: measured 16-22 us between the end of the device's work and the host's clock, against
        # 42-54 us when the end is polled for first and the synchronisation starts on an idle GPU)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ev0.elapsed_time(ev1)   # host wall seconds, device ms (events on the launch stream)

    # The paper's own protocol (section 6: 5 warm-up launches, mean of 10 timed ones), first thing
    # in the process, before the clock governor has seen any load: reported beside the sustained figure.
    cold_wall, cold_ms = timed(5, 10)
    cold = {"protocol": "5 warm-up + 10 timed launches, no clock ramp, first work of the process",
            "ms_per_step": round(cold_wall * 1e3 / 10, 5), "launch_us": round(cold_ms * 1e3 / 10, 2),
            "value": round(w.flops / (cold_wall / 10) / 1e12, 2), "unit": "TFLOP/s"}
    probe = None
    if args.mfma_probe and w.name != "cfg5_batched_512" and w.name != "cfg1_256_rowrow_f32":
        es_k = 32 if w.ab_dtype == "f32" else 64
        probe, probe_step = mfma_probe(w.ab_dtype, max(1, w.K // es_k // max(1, plan.split_k)), args.ramp_seconds)

    ramp_launches = clock_ramp(step, args.ramp_seconds)
    wall, dev_ms = timed(args.warmup, args.steps)

    in_kernel = None
    if plan.kernel == 2:
        # A few launches more, with time stamps from inside the kernel (prism_gemm_batched_stamped):
        # how long the phases of a workgroup take and which shader clock the GPU sustains in the K loop.
        stamps = torch.zeros(plan.workgroups * P.STAMP_BYTES_PER_WORKGROUP // 8, dtype=torch.int64, device="cuda")
        for _ in range(3):
            status = P.prism_gemm_batched_stamped(*call[:-1], stamps, stamps.numel() * 8, stream.cuda_stream)
            assert status == 0, status
        torch.cuda.synchronize()
        st = stamps.cpu().numpy().reshape(-1, 4, 2).astype(np.float64)    # [workgroup, point, (cycles, 100 MHz ticks)]
        d_cyc, d_us = np.diff(st[:, :, 0], axis=1), np.diff(st[:, :, 1], axis=1) / 100.0
        k_steps = (w.K // (32 if w.ab_dtype == "f32" else 64)) / max(1, plan.split_k)
        loop_clock = d_cyc[:, 1].sum() / d_us[:, 1].sum()
        die_clock = [d_cyc[g::8, 1].sum() / d_us[g::8, 1].sum() for g in range(8) if st[g::8].size]
        in_kernel = {
            "k_loop_clock_mhz": round(loop_clock, 0), "k_loop_cycles_per_step": round(d_cyc[:, 1].mean() / k_steps, 1),
            "k_loop_us_per_step": round(d_us[:, 1].mean() / k_steps, 4),
            "us_entry_to_first_fragments": round(d_us[:, 0].mean(), 2), "us_k_loop": round(d_us[:, 1].mean(), 2),
            "us_epilogue": round(d_us[:, 2].mean(), 2),
            "us_first_entry_to_last_end": round((st[:, 3, 1].max() - st[:, 0, 1].min()) / 100.0, 2),
            "die_k_loop_clock_mhz": [round(c, 0) for c in die_clock],
            "peak_at_k_loop_clock_tflops": round(loop_clock * 1e6 * 256 * (256 if w.ab_dtype == "f32" else 4096) / 1e12, 1),
            "what": "per-workgroup averages of one stamped launch; the peak at the K loop's clock is 256 compute units "
                    "x FLOP per clock x the clock measured inside the K loop",
        }
        if plan.workgroups <= 256:   # one round of workgroups: every K loop runs at the same time
            loop_tflops = w.flops / (d_us[:, 1].mean() * 1e-6) / 1e12
            in_kernel["k_loop_tflops"] = round(loop_tflops, 1)
            in_kernel["k_loop_frac_of_peak_at_its_clock"] = round(loop_tflops / in_kernel["peak_at_k_loop_clock_tflops"], 4)

    ms_per_step = wall * 1e3 / args.steps
    tflops = w.flops / (ms_per_step * 1e-3) / 1e12
    launch_ms = dev_ms / args.steps                 # average duration of one launch of the path
    mfma_bound = w.name != "cfg5_batched_512"
    peak_mfma = PEAK_MFMA_F32_TFLOPS if w.ab_dtype == "f32" else PEAK_MFMA_TFLOPS
    if mfma_bound:
        achieved = w.flops / (launch_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak_mfma,
                    "unit": "TFLOP/s", "frac": round(achieved / peak_mfma, 4), "traffic": None}
    else:
        achieved = algorithmic_bytes(w) / (launch_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None,
                    "device_copy_gbs": round(copy_ceiling_gbs(), 1)}
    if probe is not None:
        roofline["mfma_probe_tflops"] = probe["tflops_loop"]
        roofline["mfma_probe_clock_mhz"] = probe["clock_mhz"]
        roofline["frac_of_probe"] = round(achieved / probe["tflops_loop"], 4)
    roofline["kernel"] = {1: "gemm_staged", 2: "gemm_pipelined", 3: "gemm_persistent"}.get(plan.kernel, "none")
    roofline["launch_us"] = round(launch_ms * 1e3, 2)
    measured = MEASURED_TRAFFIC.get(w.name)
    if measured and measured[1] == source_digest():
        roofline["traffic"] = measured[0]

    out = {
        "metric": {"f32": "fp32 GEMM TFLOP/s and % of MI355X fp32 MFMA peak (1 GPU)",
                   "f16": "fp16 GEMM TFLOP/s and % of MI355X dense fp16 MFMA peak (1 GPU)",
                   "bf16": "bf16 GEMM TFLOP/s and % of MI355X dense bf16 MFMA peak (1 GPU)"}[w.ab_dtype],
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": w.ab_dtype, "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "batch": w.batch,
                   "layout": f"A {w.layout_a}, B {w.layout_b}, C row", "c_dtype": w.c_dtype,
                   "tile": f"{plan.tile_m}x{plan.tile_n}x{plan.tile_k}", "waves": plan.waves,
                   "split_k": plan.split_k, "workgroups": plan.workgroups},
        "pct_of_mfma_peak": round(100.0 * tflops / peak_mfma, 2),
        "roofline": roofline,
        "clock_ramp": {"seconds": args.ramp_seconds, "launches": ramp_launches},
        "cold": cold,
    }
    if probe is not None:
        out["mfma_probe"] = probe
    if in_kernel is not None:
        out["in_kernel"] = in_kernel
    if args.power:   # after everything that is timed, so that seconds of full load do not precede it
        power = socket_power(step, 3.0)
        if power is not None:
            out["power"] = power
        if probe is not None:   # and what the package draws with the matrix pipes alone at work
            reading = socket_power(probe_step, 2.0)
            if reading is not None:
                out["mfma_probe"]["socket_power_w"] = reading["socket_power_w"]
    if plan.split_k > 1:
        # A K split also moves the fp32 partial sums: written once by the slices, read once by
        # the reduction.  With them counted the path is bound by memory, not by the matrix pipe.
        ws_traffic = 2.0 * plan.split_k * w.batch * w.M * w.N * 4
        hbm = (algorithmic_bytes(w) + ws_traffic) / (launch_ms * 1e-3) / 1e9
        out["roofline_hbm"] = {"bound": "hbm", "achieved": round(hbm, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": round(hbm / PEAK_HBM_GBS, 4),
                               "bytes": int(algorithmic_bytes(w) + ws_traffic),
                               "what": "operands and result once, plus the split-K partial sums written and read once"}

    if not args.no_cpu_baseline:
        # the oracle as it stands, on an evenly spread subset of output rows of problem 0
        from oracle import gemm_ref, oracle_threads, decode_output, check_against_oracle
        n_rows = min(args.cpu_rows, w.M)
        rows = np.unique(np.linspace(0, w.M - 1, n_rows).astype(np.int64))
        c_in = None
        if w.beta != 0.0:   # one more call from the stated initial C, so that the sample has a defined input
            C.copy_(C_in)
            step()
            torch.cuda.synchronize()
            c_in = inp["C_in"][0].astype(np.float64)

        def oracle(b):
            return gemm_ref(inp["A"][b], inp["B"][b], ab_dtype=w.ab_dtype, M=w.M, N=w.N, K=w.K,
                            layout_a=w.layout_a, layout_b=w.layout_b, alpha=w.alpha, beta=w.beta,
                            bias=inp["bias"], c_in=c_in, rows=rows)

        # problem 0 is checked against the GPU result; small problems are too short to time
        # once, so the oracle goes on over further problems of the batch (or repeats the only
        # one) until about a second has passed
        t0 = time.perf_counter()
        ref, mag = oracle(0)
        calls = 1
        limit = w.batch if w.batch > 1 else 512
        while time.perf_counter() - t0 < 1.0 and calls < limit:
            oracle(calls % w.batch)
            calls += 1
        cpu_s = time.perf_counter() - t0
        got = C.cpu().numpy()
        got = got if w.c_dtype == "f32" else got.view(np.uint16)
        got = got.reshape(w.batch, w.M, w.N)[0][rows]
        res = check_against_oracle(decode_output(got, w.c_dtype), ref, mag, w.K, w.c_dtype)
        what = "problem 0" if calls == 1 else (f"{calls} problems of the batch" if w.batch > 1 else f"problem 0, {calls} times")
        out["cpu_baseline"] = {
            "value": round(2.0 * calls * rows.size * w.N * w.K / cpu_s / 1e12, 5), "unit": "TFLOP/s",
            "cores": oracle_threads(), "kind": "oracle",
            "sample": f"{rows.size} of {w.M} output rows x all {w.N} columns of {what}, {cpu_s:.2f} s wall",
        }
        out["parity_on_sample"] = {"ok": res["ok"], "max_err_over_bound": round(res["max_err_over_bound"], 4)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
