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
