"""Builds libprism_gemm.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libprism_gemm.so")
# the same library with a workgroup barrier after every LDS phase of the main loops (race check:
# its results must equal the normal build's bit for bit)
PARANOID_LIB_PATH = os.path.join(_HERE, "libprism_gemm_paranoid.so")
_UNITS = ["kernels.hip", "host_api.hip", "scan.hip", "probe.hip"]
_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # keep the compiler from forming packed fp32 vector ops out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _sources():
    out = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if not f.endswith(".o")]
    out.append(os.path.join(os.path.dirname(_HERE), "include", "prism_gemm.h"))
    out.append(os.path.join(os.path.dirname(_HERE), "include", "prism_scan.h"))
    return out


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH) or not os.path.exists(PARANOID_LIB_PATH):
        return True
    t = min(os.path.getmtime(LIB_PATH), os.path.getmtime(PARANOID_LIB_PATH))
    return any(os.path.getmtime(s) > t for s in _sources())


def build(force: bool = False, verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library.  Returns its path."""
    if not force and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = [os.path.join(CSRC, u.replace(".hip", ".o")) for u in _UNITS]
    paranoid_obj = os.path.join(CSRC, "kernels_paranoid.o")

    def compile_one(pair):
        src, obj = pair
        extra = ["-DPRISM_PARANOID_BARRIERS"] if obj == paranoid_obj else []
        cmd = [hipcc, *_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")

    with ThreadPoolExecutor(max_workers=len(_UNITS) + 1) as ex:
        list(ex.map(compile_one, list(zip(_UNITS, objs)) + [("kernels.hip", paranoid_obj)]))
    for lib, these in ((LIB_PATH, objs), (PARANOID_LIB_PATH, [paranoid_obj if o.endswith("kernels.o") else o for o in objs])):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *these, "-o", lib]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB_PATH


if __name__ == "__main__":
    print(build(force=True, verbose=True))
