"""Compile-time perspective tokens (csrc/persp.hpp): the cases under tests/perspective_cases
named ok_* must compile for gfx950, those named fail_* must be rejected by the compiler with
the diagnostic named in their EXPECT line.  Front end only (-fsyntax-only): no GPU needed."""
import glob
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CASES = sorted(glob.glob(os.path.join(ROOT, "tests", "perspective_cases", "*.hip")))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _compile(path):
    cmd = [HIPCC, "--offload-arch=gfx950", "-std=c++17", "-fsyntax-only", "--cuda-device-only",
           "-I", os.path.join(ROOT, "paper_2511_11939_amd", "csrc"), path]
    return subprocess.run(cmd, capture_output=True, text=True)


def test_cases_exist():
    names = [os.path.basename(c) for c in CASES]
    assert any(n.startswith("ok_") for n in names) and sum(n.startswith("fail_") for n in names) >= 5


@pytest.mark.parametrize("path", CASES, ids=[os.path.basename(c) for c in CASES])
def test_perspective_case(path):
    r = _compile(path)
    name = os.path.basename(path)
    if name.startswith("ok_"):
        assert r.returncode == 0, r.stderr
        return
    expect = re.search(r"// EXPECT: (.*)", open(path).read()).group(1).strip()
    assert r.returncode != 0, f"{name} compiled but must not"
    assert expect in r.stderr, f"{name}: expected diagnostic {expect!r} in:\n{r.stderr}"
