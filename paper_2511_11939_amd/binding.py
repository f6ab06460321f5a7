"""ctypes binding of libprism_gemm.so.  Same names as the C entry points; the
functions marshal arguments and nothing else.  `gemm` is a convenience wrapper
for torch tensors (torch supplies device memory and the stream only)."""
from __future__ import annotations

import ctypes
import enum
import os
from typing import Optional

from . import build as _build

_lib = None


class Status(enum.IntEnum):
    OK = 0
    INVALID_ARG = 1
    UNSUPPORTED = 2
    WORKSPACE = 3
    LAUNCH = 4


class DType(enum.IntEnum):
    BF16 = 0
    F16 = 1
    F32 = 2


class Layout(enum.IntEnum):
    ROW = 0
    COL = 1


_DTYPE_NAMES = {"bf16": DType.BF16, "f16": DType.F16, "f32": DType.F32}
_LAYOUT_NAMES = {"row": Layout.ROW, "col": Layout.COL}


class PrismError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = Status(status) if status in Status._value2member_map_ else status
        super().__init__(f"{where}: {prism_status_string(status)}")


class GemmDesc(ctypes.Structure):
    _fields_ = [
        ("ab_dtype", ctypes.c_int32), ("c_dtype", ctypes.c_int32),
        ("layout_a", ctypes.c_int32), ("layout_b", ctypes.c_int32), ("layout_c", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("beta", ctypes.c_float),
        ("bias", ctypes.c_void_p),
        ("split_k", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


class GemmPlan(ctypes.Structure):
    _fields_ = [
        ("kernel", ctypes.c_int32),
        ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32), ("tile_k", ctypes.c_int32),
        ("waves", ctypes.c_int32), ("split_k", ctypes.c_int32), ("swapped", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("tiles_m", ctypes.c_int64), ("tiles_n", ctypes.c_int64), ("workgroups", ctypes.c_int64),
        ("workspace_bytes", ctypes.c_size_t),
    ]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_ if n != "reserved"}


def library_path() -> str:
    return _build.LIB_PATH


def load_library():
    """Loads the built shared library; builds it first only if it does not exist.
    Raises if it can be neither found nor built -- there is no other code path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build()
    elif _build.is_stale():
        import warnings
        warnings.warn("libprism_gemm.so is older than its sources: run paper_2511_11939_amd.build.build(force=True)")
    lib = ctypes.CDLL(_build.LIB_PATH)
    i64, vp, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    dp = ctypes.POINTER(GemmDesc)
    lib.prism_gemm.argtypes = [dp, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
    lib.prism_gemm.restype = ctypes.c_int
    lib.prism_gemm_batched.argtypes = [dp, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, i64, vp]
    lib.prism_gemm_batched.restype = ctypes.c_int
    lib.prism_gemm_batched_stamped.argtypes = [dp, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, i64, vp, sz, vp]
    lib.prism_gemm_batched_stamped.restype = ctypes.c_int
    lib.prism_gemm_workspace_size.argtypes = [dp, i64, i64, i64, i64, ctypes.POINTER(sz)]
    lib.prism_gemm_workspace_size.restype = ctypes.c_int
    lib.prism_gemm_plan.argtypes = [dp, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, i64,
                                    ctypes.POINTER(GemmPlan)]
    lib.prism_gemm_plan.restype = ctypes.c_int
    lib.prism_sched_map.argtypes = [i64, i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                    ctypes.POINTER(i64)]
    lib.prism_sched_map.restype = ctypes.c_int
    lib.prism_status_string.argtypes = [ctypes.c_int]
    lib.prism_status_string.restype = ctypes.c_char_p
    lib.prism_version.restype = ctypes.c_int
    lib.prism_scan_workspace_size.argtypes = [i64, ctypes.POINTER(sz)]
    lib.prism_scan_workspace_size.restype = ctypes.c_int
    lib.prism_scan_u32.argtypes = [vp, vp, i64, vp, sz, vp]
    lib.prism_scan_u32.restype = ctypes.c_int
    lib.prism_scan_check.argtypes = [vp, vp]
    lib.prism_scan_check.restype = ctypes.c_int
    lib.prism_mfma_probe.argtypes = [ctypes.c_int32, vp, sz, ctypes.c_int32, vp, sz, vp]
    lib.prism_mfma_probe.restype = ctypes.c_int
    lib.prism_reread_environment.argtypes = []
    lib.prism_reread_environment.restype = None
    lib.prism_layout_probe.argtypes = [ctypes.c_int32, vp, vp, vp, vp]
    lib.prism_layout_probe.restype = ctypes.c_int
    lib.prism_scan_u32_static.argtypes = [vp, vp, i64, vp, vp]
    lib.prism_scan_u32_static.restype = ctypes.c_int
    _lib = lib
    return lib


def _p(x) -> Optional[int]:
    """device pointer from an int, None, or anything with data_ptr()."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _descp(d: Optional[GemmDesc]):
    return None if d is None else ctypes.byref(d)


# ---- the C entry points, same names, returning the status code -----------------------------

def prism_gemm(desc, M, N, K, A, lda, B, ldb, C, ldc, hip_stream=None) -> int:
    return load_library().prism_gemm(_descp(desc), M, N, K, _p(A), lda, _p(B), ldb, _p(C), ldc,
                                     _p(hip_stream))


def prism_gemm_batched(desc, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch,
                       hip_stream=None) -> int:
    return load_library().prism_gemm_batched(_descp(desc), M, N, K, _p(A), lda, strideA, _p(B), ldb,
                                             strideB, _p(C), ldc, strideC, batch, _p(hip_stream))


STAMP_BYTES_PER_WORKGROUP = 64


def prism_gemm_batched_stamped(desc, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch,
                               stamps, stamp_bytes, hip_stream=None) -> int:
    return load_library().prism_gemm_batched_stamped(_descp(desc), M, N, K, _p(A), lda, strideA, _p(B), ldb,
                                                     strideB, _p(C), ldc, strideC, batch, _p(stamps), stamp_bytes,
                                                     _p(hip_stream))


def prism_gemm_workspace_size(desc, M, N, K, batch=1):
    """Returns (status, bytes)."""
    out = ctypes.c_size_t(0)
    s = load_library().prism_gemm_workspace_size(_descp(desc), M, N, K, batch, ctypes.byref(out))
    return s, out.value


def prism_gemm_plan(desc, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch):
    """Returns (status, GemmPlan)."""
    plan = GemmPlan()
    s = load_library().prism_gemm_plan(_descp(desc), M, N, K, _p(A), lda, strideA, _p(B), ldb, strideB,
                                       _p(C), ldc, strideC, batch, ctypes.byref(plan))
    return s, plan


def prism_sched_map(wg, tiles_m, tiles_n, units):
    """Returns (status, tile_m, tile_n, unit)."""
    tm, tn, u = ctypes.c_int64(-1), ctypes.c_int64(-1), ctypes.c_int64(-1)
    s = load_library().prism_sched_map(wg, tiles_m, tiles_n, units, ctypes.byref(tm), ctypes.byref(tn),
                                       ctypes.byref(u))
    return s, tm.value, tn.value, u.value


MFMA_PROBE_OPERAND_BYTES = 33554432
MFMA_PROBE_COUNTER_BYTES = 32768
MFMA_PROBE_FLOP_PER_ITERATION = 2147483648.0


def prism_mfma_probe(ab_dtype, operands, operand_bytes, iterations, counters, counter_bytes, hip_stream=None) -> int:
    return load_library().prism_mfma_probe(int(ab_dtype), _p(operands), operand_bytes, iterations, _p(counters),
                                           counter_bytes, _p(hip_stream))


LAYOUT_ACCUMULATOR_BF16, LAYOUT_ACCUMULATOR_F16, LAYOUT_K_ROWS_READ = 0, 1, 2


def prism_layout_probe(what, in0, in1, out, hip_stream=None) -> int:
    return load_library().prism_layout_probe(int(what), _p(in0), _p(in1), _p(out), _p(hip_stream))


def prism_status_string(status: int) -> str:
    return load_library().prism_status_string(int(status)).decode()


def prism_version() -> int:
    return load_library().prism_version()


def prism_reread_environment() -> None:
    load_library().prism_reread_environment()


# ---- convenience for torch tensors ----------------------------------------------------------

def make_desc(ab_dtype="bf16", c_dtype="bf16", layout_a="row", layout_b="col", layout_c="row",
              alpha=1.0, beta=0.0, bias=None, split_k=0, workspace=None, workspace_bytes=None) -> GemmDesc:
    d = GemmDesc()
    d.ab_dtype = int(_DTYPE_NAMES.get(ab_dtype, ab_dtype))
    d.c_dtype = int(_DTYPE_NAMES.get(c_dtype, c_dtype))
    d.layout_a = int(_LAYOUT_NAMES.get(layout_a, layout_a))
    d.layout_b = int(_LAYOUT_NAMES.get(layout_b, layout_b))
    d.layout_c = int(_LAYOUT_NAMES.get(layout_c, layout_c))
    d.alpha, d.beta = float(alpha), float(beta)
    d.bias = _p(bias)
    d.split_k = int(split_k)
    d.reserved = 0
    d.workspace = _p(workspace)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if hasattr(workspace, "numel") else 0
    d.workspace_bytes = int(workspace_bytes)
    return d


def gemm(A, B, C, *, M, N, K, desc: GemmDesc, lda=None, ldb=None, ldc=None, batch=1,
         strideA=None, strideB=None, strideC=None, stream=None):
    """Enqueue C <- alpha*A*B + bias + beta*C on `stream` (a torch.cuda.Stream, a raw
    hipStream_t value or None for torch's current stream).  A, B, C: device tensors or
    raw device pointers, laid out as `desc` says.  Raises PrismError on a bad status."""
    if lda is None:
        lda = K if desc.layout_a == Layout.ROW else M
    if ldb is None:
        ldb = N if desc.layout_b == Layout.ROW else K
    if ldc is None:
        ldc = N if desc.layout_c == Layout.ROW else M
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    if batch == 1 and strideA is None and strideB is None and strideC is None:
        s = prism_gemm(desc, M, N, K, A, max(lda, 1), B, max(ldb, 1), C, max(ldc, 1), stream)
    else:
        strideA = M * K if strideA is None else strideA
        strideB = K * N if strideB is None else strideB
        strideC = M * N if strideC is None else strideC
        s = prism_gemm_batched(desc, M, N, K, A, max(lda, 1), strideA, B, max(ldb, 1), strideB,
                               C, max(ldc, 1), strideC, batch, stream)
    if s != Status.OK:
        raise PrismError(s, "prism_gemm")


# ---- prefix scan (include/prism_scan.h) ------------------------------------------------------

def prism_scan_workspace_size(n):
    out = ctypes.c_size_t(0)
    s = load_library().prism_scan_workspace_size(n, ctypes.byref(out))
    return s, out.value


def prism_scan_u32(inp, out, n, workspace, workspace_bytes, hip_stream=None) -> int:
    return load_library().prism_scan_u32(_p(inp), _p(out), n, _p(workspace), workspace_bytes, _p(hip_stream))


def prism_scan_check(workspace, hip_stream=None) -> int:
    return load_library().prism_scan_check(_p(workspace), _p(hip_stream))


def prism_scan_u32_static(inp, out, n, gave_up=None, hip_stream=None) -> int:
    return load_library().prism_scan_u32_static(_p(inp), _p(out), n, _p(gave_up), _p(hip_stream))


def scan_u32(inp, out, n, workspace, *, stream=None):
    """Enqueue the inclusive uint32 prefix sum of `inp` into `out` (may be the same tensor) on
    `stream` (torch stream, raw hipStream_t or None for torch's current stream).  `workspace`:
    a device tensor of at least prism_scan_workspace_size(n) bytes.  Raises on a bad status."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    s = prism_scan_u32(inp, out, n, workspace, nbytes, stream)
    if s != Status.OK:
        raise PrismError(s, "prism_scan_u32")
