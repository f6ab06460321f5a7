"""Helpers for the GPU parity tests: run a workload through the C ABI (via the
Python binding) and compare with the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2511_11939_amd as P
from oracle import gemm_ref, decode_output, check_against_oracle
from workloads import GemmWorkload, make_inputs

ESIZE = {"bf16": 2, "f16": 2, "f32": 4}


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> device int16 tensor with the same bytes; float32 stays float32."""
    bits = np.ascontiguousarray(bits)
    return torch.from_numpy(bits if bits.dtype == np.float32 else bits.view(np.int16)).cuda()


def alloc_c(n_elems: int, c_dtype: str, fill=None) -> torch.Tensor:
    dt = torch.float32 if c_dtype == "f32" else torch.int16
    t = torch.empty(n_elems, dtype=dt, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def c_to_numpy(c: torch.Tensor, c_dtype: str) -> np.ndarray:
    a = c.cpu().numpy()
    return a if c_dtype == "f32" else a.view(np.uint16)


def workspace_for(desc, M, N, K, batch=1):
    s, nbytes = P.prism_gemm_workspace_size(desc, M, N, K, batch)
    assert s == 0, P.prism_status_string(s)
    if nbytes == 0:
        return None
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    desc.workspace = ws.data_ptr()
    desc.workspace_bytes = nbytes
    return ws


def run_workload(w: GemmWorkload, inputs: dict, *, c_dtype=None, split_k=None, sync=True):
    """Runs w on the GPU; returns (stored C as numpy [batch, M, N], plan dict)."""
    c_dtype = c_dtype or w.c_dtype
    A, B = to_dev(inputs["A"]), to_dev(inputs["B"])
    bias = None if inputs.get("bias") is None else torch.from_numpy(inputs["bias"]).cuda()
    C = alloc_c(w.batch * w.M * w.N, c_dtype)
    if w.beta != 0.0:
        assert c_dtype == "f32", "workloads with beta keep C in fp32"
        C.copy_(torch.from_numpy(inputs["C_in"].ravel()))
    desc = P.make_desc(ab_dtype=w.ab_dtype, c_dtype=c_dtype, layout_a=w.layout_a, layout_b=w.layout_b,
                       alpha=w.alpha, beta=w.beta, bias=bias, split_k=w.split_k if split_k is None else split_k)
    ws = workspace_for(desc, w.M, w.N, w.K, w.batch)
    s, plan = P.prism_gemm_plan(desc, w.M, w.N, w.K, A, w.lda(), w.M * w.K, B, w.ldb(), w.K * w.N,
                                C, w.N, w.M * w.N, w.batch)
    assert s == 0, P.prism_status_string(s)
    P.gemm(A, B, C, M=w.M, N=w.N, K=w.K, desc=desc, batch=w.batch,
           strideA=w.M * w.K, strideB=w.K * w.N, strideC=w.M * w.N)
    if sync:
        torch.cuda.synchronize()
    del ws
    return c_to_numpy(C, c_dtype).reshape(w.batch, w.M, w.N), plan.as_dict()


def assert_matches_oracle(w: GemmWorkload, inputs: dict, c_stored: np.ndarray, *, c_dtype=None,
                          rows=None, batch_index=0, what=""):
    """Every entry of the given rows (all rows if None) of one problem against the oracle."""
    c_dtype = c_dtype or w.c_dtype
    ref, mag = gemm_ref(inputs["A"][batch_index], inputs["B"][batch_index], ab_dtype=w.ab_dtype,
                        M=w.M, N=w.N, K=w.K, layout_a=w.layout_a, layout_b=w.layout_b,
                        alpha=w.alpha, beta=w.beta, bias=inputs.get("bias"), rows=rows,
                        c_in=None if w.beta == 0.0 else inputs["C_in"][batch_index].astype(np.float64))
    got = c_stored[batch_index]
    if rows is not None:
        got = got[np.asarray(rows)]
    res = check_against_oracle(decode_output(got, c_dtype), ref, mag, w.K, c_dtype)
    assert res["ok"], f"{w.name} {what}: {res}"
    return res


def assert_every_entry_matches_oracle(w: GemmWorkload, inputs: dict, c_stored: np.ndarray, *, c_dtype=None,
                                      batch_index=0, block=2048, what=""):
    """All rows of one problem against the oracle, a block of rows at a time (the oracle's fp64
    outputs of a whole 16384 x 4096 result would take a gigabyte)."""
    worst = 0.0
    for r0 in range(0, w.M, block):
        rows = np.arange(r0, min(r0 + block, w.M))
        res = assert_matches_oracle(w, inputs, c_stored, c_dtype=c_dtype, rows=rows, batch_index=batch_index,
                                    what=f"{what} rows {r0}..{rows[-1]}")
        worst = max(worst, res["max_err_over_bound"])
    return worst


def tile_probe_rows(M: int, tile: int = 256, per_tile=(0, 1, 31, 32, 63, 64, 100, 127, 128, 191, 200, 255)):
    """Row indices that touch every workgroup tile row, every wave row and both
    halves of the 32-row MFMA blocks."""
    rows = sorted({t + r for t in range(0, M, tile) for r in per_tile if t + r < M})
    return rows
