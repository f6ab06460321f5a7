"""The benchmark's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figures_are_tied_to_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    digest = bench.source_digest()
    assert len(digest) == 16
    for name, (nbytes, tag) in bench.MEASURED_TRAFFIC.items():
        assert nbytes > 0 and len(tag) == 16, name


def test_the_source_digest_does_not_change_with_a_rebuild(tmp_path):
    """Objects and other build products next to the sources must not enter the digest: the box
    that runs the benchmark builds its own."""
    sys.path.insert(0, ROOT)
    import bench
    before = bench.source_digest()
    csrc = os.path.join(ROOT, "paper_2511_11939_amd", "csrc")
    stray = [os.path.join(csrc, "zz_digest_probe.o"), os.path.join(csrc, "zz_digest_probe.tmp")]
    try:
        for f in stray:
            with open(f, "wb") as fh:
                fh.write(os.urandom(64))
        assert bench.source_digest() == before
    finally:
        for f in stray:
            if os.path.exists(f):
                os.remove(f)
    # and it does follow the sources
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(csrc, "*"))):
        if f.endswith((".hip", ".hpp")):
            h.update(os.path.basename(f).encode())
            h.update(open(f, "rb").read())
    assert before == h.hexdigest()[:16]


import json

import pytest


@pytest.mark.gpu
@pytest.mark.parametrize("workload", ["cfg2_4096_bf16", "cfg5_batched_512", "scan_u32_2p28"])
def test_bench_prints_one_json_line_with_the_contract_keys(workload):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload, "--steps", "3",
                        "--warmup", "1", "--ramp-seconds", "0.05", "--cpu-rows", "64"] +
                       ([] if workload == "cfg2_4096_bf16" else ["--no-power"]),
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["config"]["workload"] == workload and "model" not in d["config"]
    roof = d["roofline"]
    assert roof["bound"] in ("mfma", "hbm") and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["cores"] >= 1
    assert d["parity_on_sample"]["ok"] is True
    if workload == "cfg2_4096_bf16":
        # the sustained figure comes with the paper's cold protocol and the matrix-pipe ceiling
        assert d["cold"]["value"] > 0 and d["cold"]["ms_per_step"] > 0
        assert d["mfma_probe"]["tflops_loop"] > 0 and 500 < d["mfma_probe"]["clock_mhz"] < 3000
        assert roof["mfma_probe_tflops"] == d["mfma_probe"]["tflops_loop"]
        # and with the clock the K loop itself ran at, from stamps taken inside the kernel
        assert 500 < d["in_kernel"]["k_loop_clock_mhz"] < 3000 and len(d["in_kernel"]["die_k_loop_clock_mhz"]) == 8
        assert 2048 <= d["in_kernel"]["k_loop_cycles_per_step"] < 4096
        assert 0.5 < d["in_kernel"]["k_loop_frac_of_peak_at_its_clock"] <= 1.0
        # the package power, where the machine's management tool reports it
        if "power" in d:
            assert d["power"]["socket_power_w"] > 100 and d["power"]["samples"] >= 1


@pytest.mark.gpu
def test_a_k_split_reports_the_memory_roofline_too():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "cfg4_splitk_f16", "--steps", "3",
                        "--warmup", "1", "--ramp-seconds", "0.05", "--cpu-rows", "16", "--no-mfma-probe"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([ln for ln in r.stdout.splitlines() if ln.strip()][0])
    assert d["dtype"] == "f16" and d["metric"].startswith("fp16")
    if d["config"]["split_k"] > 1:
        hbm = d["roofline_hbm"]
        assert hbm["bound"] == "hbm" and abs(hbm["frac"] - hbm["achieved"] / hbm["peak"]) < 1e-3
        assert hbm["bytes"] > 132 * (1 << 20)
