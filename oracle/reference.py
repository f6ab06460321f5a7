"""ctypes front end of the C oracle (oracle/gemm_oracle.c).

Test infrastructure only: a plain fp64 triple loop for
C <- alpha*A*B + bias + beta*C  (the paper's section 6.1 definition, with the
16-bit operand types of its section 6.2 kernel or the fp32 operands of its
section 6.1 sgemm).  This module marshals
arguments; the arithmetic is all in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_SCAN_SRC = os.path.join(_HERE, "scan_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_oracle.so")
_lib = None

_DTYPE_CODE = {"bf16": 0, "f16": 1}


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over output entries)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SCAN_SRC)))
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
             "-fno-fast-math", "-ffp-contract=off", _SRC, _SCAN_SRC, "-o", _LIB, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.prism_oracle_gemm.argtypes = [
            ctypes.c_int, i64, i64, i64, vp, i64, i64, vp, i64, i64,
            dbl, dbl, vp, vp, vp, i64, vp, vp]
        lib.prism_oracle_gemm.restype = ctypes.c_int
        lib.prism_oracle_sgemm.argtypes = [
            i64, i64, i64, vp, i64, i64, vp, i64, i64,
            dbl, dbl, vp, vp, vp, i64, vp, vp]
        lib.prism_oracle_sgemm.restype = ctypes.c_int
        lib.prism_oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        lib.prism_oracle_decode_bf16.restype = dbl
        lib.prism_oracle_decode_f16.argtypes = [ctypes.c_uint16]
        lib.prism_oracle_decode_f16.restype = dbl
        lib.prism_oracle_threads.restype = ctypes.c_int
        lib.prism_oracle_inclusive_scan_u32.argtypes = [vp, vp, i64]
        lib.prism_oracle_inclusive_scan_u32.restype = ctypes.c_int
        _lib = lib
    return _lib


def oracle_threads() -> int:
    return int(_load().prism_oracle_threads())


def decode_bits(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Decode uint16 bit patterns to float64 with the oracle's own decoders."""
    lib = _load()
    f = lib.prism_oracle_decode_bf16 if dtype == "bf16" else lib.prism_oracle_decode_f16
    table = np.array([f(h) for h in range(65536)], dtype=np.float64)
    return table[np.asarray(bits, dtype=np.uint16)]


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def gemm_ref(A: np.ndarray, B: np.ndarray, *, ab_dtype: str, M: int, N: int, K: int,
             layout_a: str = "row", layout_b: str = "col",
             lda: Optional[int] = None, ldb: Optional[int] = None,
             alpha: float = 1.0, beta: float = 0.0,
             bias: Optional[np.ndarray] = None, c_in: Optional[np.ndarray] = None,
             rows: Optional[Sequence[int]] = None):
    """One GEMM.  A, B: uint16 bit patterns as stored, or float32 values when
    ab_dtype is "f32" (any shape; read flat with the given leading dimensions).
    c_in: float64 [M, N] (already decoded).
    Returns (ref, mag), float64 arrays of shape [len(rows) or M, N].
    """
    store = np.float32 if ab_dtype == "f32" else np.uint16
    assert np.asarray(A).dtype == store and np.asarray(B).dtype == store, "operands must be stored as " + str(store)
    A = np.ascontiguousarray(A).reshape(-1)
    B = np.ascontiguousarray(B).reshape(-1)
    if lda is None:
        lda = K if layout_a == "row" else M
    if ldb is None:
        ldb = N if layout_b == "row" else K
    a_si, a_sk = (lda, 1) if layout_a == "row" else (1, lda)
    b_sk, b_sj = (ldb, 1) if layout_b == "row" else (1, ldb)
    if M > 0 and K > 0:
        assert A.size > (M - 1) * a_si + (K - 1) * a_sk, "A too small"
    if N > 0 and K > 0:
        assert B.size > (K - 1) * b_sk + (N - 1) * b_sj, "B too small"
    if rows is None:
        rows_arr, n_rows = None, M
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        n_rows = rows_arr.size
        assert n_rows == 0 or (rows_arr.min() >= 0 and rows_arr.max() < M)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.size == N
    if c_in is not None:
        c_in = np.ascontiguousarray(c_in, dtype=np.float64)
        assert c_in.shape == (M, N)
    ref = np.empty((n_rows, N), dtype=np.float64)
    mag = np.empty((n_rows, N), dtype=np.float64)
    tail = (_ptr(A), a_si, a_sk, _ptr(B), b_sk, b_sj, float(alpha), float(beta), _ptr(bias), _ptr(c_in),
            _ptr(rows_arr), n_rows, _ptr(ref), _ptr(mag))
    if ab_dtype == "f32":
        rc = _load().prism_oracle_sgemm(M, N, K, *tail)
    else:
        rc = _load().prism_oracle_gemm(_DTYPE_CODE[ab_dtype], M, N, K, *tail)
    if rc != 0:
        raise ValueError("the oracle rejected its arguments")
    return ref, mag


def gemm_ref_workload(w, inputs: dict, *, batch_index: int = 0,
                      rows: Optional[Sequence[int]] = None):
    """Oracle result for one problem of a workloads.GemmWorkload."""
    return gemm_ref(inputs["A"][batch_index], inputs["B"][batch_index],
                    ab_dtype=w.ab_dtype, M=w.M, N=w.N, K=w.K,
                    layout_a=w.layout_a, layout_b=w.layout_b,
                    alpha=w.alpha, beta=w.beta, bias=inputs.get("bias"), rows=rows,
                    c_in=None if w.beta == 0.0 else inputs["C_in"][batch_index].astype(np.float64))


def inclusive_scan_u32_ref(x: np.ndarray) -> np.ndarray:
    """Inclusive prefix sum modulo 2^32 of a uint32 array (the C oracle's running sum)."""
    x = np.ascontiguousarray(x)
    assert x.dtype == np.uint32 and x.ndim == 1
    out = np.empty_like(x)
    rc = _load().prism_oracle_inclusive_scan_u32(_ptr(x), _ptr(out), x.size)
    if rc != 0:
        raise ValueError("the oracle rejected its arguments")
    return out
