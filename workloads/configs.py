"""The synthetic GEMM workloads and how their operands are laid out.

Storage convention (shared by every consumer): A is the logical M x K matrix,
B the logical K x N matrix, C the logical M x N matrix.  "row" means the last
logical index is contiguous, "col" means the first one is.  A batched workload
stores its problems back to back with no padding.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

from . import generators as g


@dataclass(frozen=True)
class GemmWorkload:
    name: str
    M: int
    N: int
    K: int
    batch: int = 1
    ab_dtype: str = "bf16"          # "bf16" | "f16" | "f32"
    c_dtype: str = "f32"            # "bf16" | "f16" | "f32"
    layout_a: str = "row"
    layout_b: str = "col"
    dist_a: Tuple = ("normal", 1.0)  # ("normal", sigma) | ("uniform",) | ("ints", lo, hi)
    dist_b: Tuple = ("normal", 1.0)
    bias: bool = False
    alpha: float = 1.0
    beta: float = 0.0               # != 0: C holds N(0, 1) values (tensor 3) before the call
    split_k: int = 0                # 0 = library decides, 1 = off, n = forced
    seed: int = 0x5EED0000

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K * self.batch

    def lda(self) -> int:
        return self.K if self.layout_a == "row" else self.M

    def ldb(self) -> int:
        return self.N if self.layout_b == "row" else self.K

    def with_(self, **kw) -> "GemmWorkload":
        return replace(self, **kw)


CONFIGS = {
    # small case: both operands row-major, fp32 output
    "cfg1_256_rowrow_f32": GemmWorkload(
        "cfg1_256_rowrow_f32", 256, 256, 256, ab_dtype="bf16", c_dtype="f32",
        layout_a="row", layout_b="row", dist_a=("uniform",), dist_b=("uniform",),
        seed=0x5EED0001),
    # headline square case
    "cfg2_4096_bf16": GemmWorkload(
        "cfg2_4096_bf16", 4096, 4096, 4096, ab_dtype="bf16", c_dtype="bf16",
        seed=0x5EED0002),
    # projection-shaped: tokens x hidden, weights N(0, 0.02), fused bias
    "cfg3_proj_bias": GemmWorkload(
        "cfg3_proj_bias", 16384, 4096, 4096, ab_dtype="bf16", c_dtype="bf16",
        dist_b=("normal", 0.02), bias=True, seed=0x5EED0003),
    # skinny, long K, fp16, split-K with on-device reduction
    "cfg4_splitk_f16": GemmWorkload(
        "cfg4_splitk_f16", 1024, 1024, 32768, ab_dtype="f16", c_dtype="f32",
        dist_a=("uniform",), dist_b=("uniform",), seed=0x5EED0004),
    # many small independent problems
    "cfg5_batched_512": GemmWorkload(
        "cfg5_batched_512", 512, 512, 512, batch=256, ab_dtype="bf16", c_dtype="bf16",
        seed=0x5EED0005),
    # fp32 sgemm, every matrix row-major, both scalars in use
    "sgemm_4096_rowrow": GemmWorkload(
        "sgemm_4096_rowrow", 4096, 4096, 4096, ab_dtype="f32", c_dtype="f32",
        layout_a="row", layout_b="row", dist_a=("uniform",), dist_b=("uniform",),
        alpha=1.5, beta=0.5, seed=0x5EED0006),
}


def _draw(dist: Tuple, seed: int, tensor_id: int, n: int) -> np.ndarray:
    kind = dist[0]
    if kind == "uniform":
        return g.uniform_pm1(seed, tensor_id, n)
    if kind == "normal":
        return g.normal(seed, tensor_id, n, dist[1])
    if kind == "ints":
        return g.small_integers(seed, tensor_id, n, dist[1], dist[2])
    if kind == "ones":
        return np.ones(n, dtype=np.float32)
    raise ValueError(kind)


def _store(x: np.ndarray, batch: int, rows: int, cols: int, layout: str) -> np.ndarray:
    """x holds batch*rows*cols logical row-major values; return the stored array."""
    x = x.reshape(batch, rows, cols)
    if layout == "col":
        x = np.ascontiguousarray(np.swapaxes(x, 1, 2))
    return x


def make_inputs(w: GemmWorkload) -> dict:
    """Returns {"A": [batch, ...], "B": [batch, ...], "bias": float32[N] | None,
    "C_in": float32[batch, M, N] | None}.

    A is stored [batch, M, K] (row) or [batch, K, M] (col); B is stored
    [batch, K, N] (row) or [batch, N, K] (col).  Values are uint16 bit patterns of
    `w.ab_dtype`, rounded once from float32 draws, or the float32 draws themselves
    for fp32 operands.  C_in (only for beta != 0) is what C holds before the call.
    """
    a = _draw(w.dist_a, w.seed, 0, w.batch * w.M * w.K)
    b = _draw(w.dist_b, w.seed, 1, w.batch * w.K * w.N)
    A = _store(g.encode(a, w.ab_dtype), w.batch, w.M, w.K, w.layout_a)
    B = _store(g.encode(b, w.ab_dtype), w.batch, w.K, w.N, w.layout_b)
    bias: Optional[np.ndarray] = None
    if w.bias:
        bias = g.normal(w.seed, 2, w.N, 1.0)
    c_in = None
    if w.beta != 0.0:
        c_in = g.normal(w.seed, 3, w.batch * w.M * w.N, 1.0).reshape(w.batch, w.M, w.N)
    return {"A": A, "B": B, "bias": bias, "C_in": c_in}
