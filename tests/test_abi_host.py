"""Host-only checks of the C ABI: the library loads, exports what the header
declares, rejects bad arguments before any launch, and its planning and tile
scheduling arithmetic is sound.  No GPU is touched."""
import ctypes
import os
import re

import pytest

import paper_2511_11939_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
S = P.Status


def _declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("prism_gemm.h", "prism_scan.h"))
    return sorted(set(re.findall(r"PRISM_API[^;(]*?\b(prism_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"prism_gemm", "prism_gemm_batched", "prism_gemm_workspace_size", "prism_gemm_plan",
            "prism_sched_map", "prism_status_string", "prism_version",
            "prism_scan_workspace_size", "prism_scan_u32", "prism_scan_check"} <= set(names)
    lib = ctypes.CDLL(P.library_path())
    for n in names:
        assert hasattr(lib, n), n
    assert P.prism_version() >= 100
    assert P.prism_status_string(0) == "PRISM_OK"
    assert P.prism_status_string(3) == "PRISM_ERR_WORKSPACE"
    assert P.prism_status_string(99) == "PRISM_ERR_UNKNOWN"


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(P.GemmDesc) == 64
    assert P.GemmDesc.bias.offset == 32 and P.GemmDesc.workspace.offset == 48
    assert ctypes.sizeof(P.GemmPlan) == 64


FAKE = 0x7F0000000000  # a 16-byte aligned non-null address; nothing is launched in these tests


def _call(desc, M=64, N=64, K=64, A=FAKE, lda=None, B=FAKE + (1 << 30), ldb=None, C=FAKE + (2 << 30), ldc=None):
    lda = K if lda is None else lda
    ldb = K if ldb is None else ldb
    ldc = N if ldc is None else ldc
    return P.prism_gemm(desc, M, N, K, A, lda, B, ldb, C, ldc, None)


def test_argument_errors_are_reported_before_any_launch():
    d = P.make_desc()
    assert P.prism_gemm(None, 1, 1, 1, FAKE, 1, FAKE, 1, FAKE, 1, None) == S.INVALID_ARG
    assert _call(d, M=-1) == S.INVALID_ARG
    assert _call(d, K=-5, lda=1, ldb=1) == S.INVALID_ARG
    assert _call(d, A=None) == S.INVALID_ARG
    assert _call(d, B=None) == S.INVALID_ARG
    assert _call(d, C=None) == S.INVALID_ARG
    assert _call(d, lda=63) == S.INVALID_ARG          # row-major A needs lda >= K
    assert _call(d, ldb=63) == S.INVALID_ARG          # col-major B needs ldb >= K
    assert _call(d, ldc=63) == S.INVALID_ARG
    assert _call(d, C=FAKE + 64) == S.INVALID_ARG     # C overlaps A
    for field, bad in (("ab_dtype", 2), ("ab_dtype", 7), ("c_dtype", 3), ("layout_a", 2),
                       ("layout_b", -1), ("layout_c", 5)):
        e = P.make_desc()
        setattr(e, field, bad)
        assert _call(e) == S.UNSUPPORTED, field
    e = P.make_desc()
    e.reserved = 1
    assert _call(e) == S.INVALID_ARG
    e = P.make_desc(alpha=float("nan"))
    assert _call(e) == S.INVALID_ARG
    e = P.make_desc(split_k=-2)
    assert _call(e) == S.INVALID_ARG
    # forced split without / with too small a workspace
    e = P.make_desc(split_k=4)
    assert _call(e, K=1024, lda=1024, ldb=1024) == S.WORKSPACE
    e = P.make_desc(split_k=4, workspace=FAKE + (3 << 30), workspace_bytes=4 * 64 * 64 * 4 - 1)
    assert _call(e, K=1024, lda=1024, ldb=1024) == S.WORKSPACE
    # col-major operands need ld >= rows
    e = P.make_desc(layout_a="col", layout_b="row", layout_c="col")
    assert _call(e, M=80, lda=79, ldb=64, ldc=80) == S.INVALID_ARG
    assert _call(e, M=80, lda=80, ldb=63, ldc=80) == S.INVALID_ARG
    assert _call(e, M=80, lda=80, ldb=64, ldc=79) == S.INVALID_ARG


def test_empty_problems_are_ok_without_pointers():
    d = P.make_desc()
    assert P.prism_gemm(d, 0, 64, 64, None, 64, None, 64, None, 64, None) == S.OK
    assert P.prism_gemm(d, 64, 0, 64, None, 64, None, 64, None, 1, None) == S.OK
    assert P.prism_gemm_batched(d, 64, 64, 64, None, 64, 0, None, 64, 0, None, 64, 0, 0, None) == S.OK


def test_batched_c_overlap_is_rejected():
    d = P.make_desc()
    args = (d, 64, 64, 64, FAKE, 64, 4096, FAKE + (1 << 30), 64, 4096, FAKE + (2 << 30), 64)
    assert P.prism_gemm_batched(*args, 4095, 4, None) == S.INVALID_ARG
    s, plan = P.prism_gemm_plan(*args, 4096, 4)
    assert s == S.OK and plan.workgroups >= 4


def _plan(desc, M, N, K, batch=1, A=None, B=None, C=None, lda=None, ldb=None):
    lda = lda or (K if desc.layout_a == 0 else M)
    ldb = ldb or (N if desc.layout_b == 0 else K)
    ldc = N if desc.layout_c == 0 else M
    s, p = P.prism_gemm_plan(desc, M, N, K, A, lda, M * K, B, ldb, K * N, C, ldc, M * N, batch)
    assert s == S.OK
    return p


def test_plans_for_the_five_workloads():
    p = _plan(P.make_desc(layout_b="row", c_dtype="f32"), 256, 256, 256)
    assert p.kernel == 2 and p.tile_m == 128 and p.split_k == 1   # row-major B: pipeline, B kept as k-rows in LDS
    p = _plan(P.make_desc(), 4096, 4096, 4096)
    assert (p.kernel, p.tile_m, p.tile_n, p.tile_k, p.workgroups, p.split_k) == (2, 256, 256, 64, 256, 1)
    p = _plan(P.make_desc(), 16384, 4096, 4096)
    assert (p.kernel, p.workgroups, p.split_k) == (2, 1024, 1)
    p = _plan(P.make_desc(ab_dtype="f16", c_dtype="f32"), 1024, 1024, 32768)
    assert p.kernel == 2 and p.split_k > 1
    assert p.workspace_bytes == p.split_k * 1024 * 1024 * 4
    assert p.workgroups == p.tiles_m * p.tiles_n * p.split_k
    p = _plan(P.make_desc(), 512, 512, 512, batch=256)
    # many tiles with a short K loop: 256 persistent workgroups walk the 1024 tiles
    assert p.kernel == 3 and p.workgroups == 256 and p.tiles_m * p.tiles_n == 4 and p.split_k == 1


def test_plan_falls_back_to_staged_kernel():
    d = P.make_desc()
    assert _plan(d, 256, 256, 100).kernel == 1                     # K not a multiple of 64
    assert _plan(d, 256, 256, 128, A=FAKE + 2).kernel == 1         # misaligned A
    assert _plan(d, 256, 256, 128, lda=129).kernel == 1            # rows not 16-byte aligned
    # operands contiguous along m or n stay on the pipeline when whole aligned chunks exist
    pc = _plan(P.make_desc(layout_a="col"), 256, 256, 128)
    assert pc.kernel == 2 and pc.tile_m == 128
    assert _plan(P.make_desc(layout_a="col"), 252, 256, 128).kernel == 1                  # M not a multiple of 8
    assert _plan(P.make_desc(layout_a="col", layout_b="row"), 256, 256, 128).kernel == 2
    assert _plan(P.make_desc(layout_b="row"), 256, 260, 128).kernel == 1                   # N not a multiple of 8
    assert _plan(d, 256, 256, 128).kernel == 2
    # a column-major C is run as the transposed problem
    pc = _plan(P.make_desc(layout_c="col"), 320, 256, 128)
    assert pc.swapped == 1 and pc.kernel == 2 and pc.tiles_m * pc.tile_m >= 256   # M and N trade places
    assert pc.tiles_n * pc.tile_n >= 320


def test_split_k_never_leaves_an_empty_slice():
    for K in (64, 128, 1000, 4096, 32768):
        for want in (1, 2, 3, 5, 7, 64, 1000):
            d = P.make_desc(split_k=want, c_dtype="f32")
            p = _plan(d, 128, 128, K)
            ksteps = -(-K // 64)
            assert 1 <= p.split_k <= min(want, ksteps)
            per = -(-ksteps // p.split_k)
            assert (p.split_k - 1) * per < ksteps                  # the last slice has work
            s, nbytes = P.prism_gemm_workspace_size(d, 128, 128, K, 1)
            assert s == S.OK and nbytes == (p.split_k * 128 * 128 * 4 if p.split_k > 1 else 0)


@pytest.mark.parametrize("tm,tn,units", [(16, 16, 1), (64, 16, 1), (4, 4, 16), (2, 2, 256), (1, 1, 1),
                                         (3, 5, 7), (1, 37, 1), (13, 1, 3), (5, 5, 1)])
def test_scheduler_is_a_bijection(tm, tn, units):
    total = tm * tn * units
    seen = set()
    for wg in range(total):
        s, a, b, u = P.prism_sched_map(wg, tm, tn, units)
        assert s == S.OK and 0 <= a < tm and 0 <= b < tn and 0 <= u < units
        seen.add((a, b, u))
    assert len(seen) == total
    assert P.prism_sched_map(total, tm, tn, units)[0] == S.INVALID_ARG
    assert P.prism_sched_map(-1, tm, tn, units)[0] == S.INVALID_ARG


def test_scheduler_gives_each_die_a_compact_block():
    """16 x 16 tiles on 256 compute units: the 32 workgroups of one die (ids congruent mod 8)
    must share few operand panels: at most 4 tile rows and 8 tile columns."""
    for die in range(8):
        rows, cols = set(), set()
        for wg in range(die, 256, 8):
            _, a, b, _ = P.prism_sched_map(wg, 16, 16, 1)
            rows.add(a)
            cols.add(b)
        assert len(rows) <= 4 and len(cols) <= 8
    # first wave of a 64 x 16 grid (1024 tiles): the same property for the first 256 ids
    for die in range(8):
        rows, cols = set(), set()
        for wg in range(die, 256, 8):
            _, a, b, _ = P.prism_sched_map(wg, 64, 16, 1)
            rows.add(a)
            cols.add(b)
        assert len(rows) * len(cols) <= 64 and len(rows) + len(cols) <= 12


def test_fp32_operands_need_an_fp32_result():
    FAKE_A, FAKE_B, FAKE_C = FAKE, FAKE + (1 << 30), FAKE + (2 << 30)
    for cd in ("bf16", "f16"):
        d = P.make_desc(ab_dtype="f32", c_dtype=cd)
        assert P.prism_gemm(d, 64, 64, 64, FAKE_A, 64, FAKE_B, 64, FAKE_C, 64, None) == S.UNSUPPORTED
    d = P.make_desc(ab_dtype="f32", c_dtype="f32", layout_b="row")
    s, plan = P.prism_gemm_plan(d, 4096, 4096, 4096, None, 4096, 0, None, 4096, 0, None, 4096, 0, 1)
    assert s == S.OK and plan.kernel == 2 and plan.tile_m == 128 and plan.tile_k == 32 and plan.workgroups == 32 * 32
    s, plan = P.prism_gemm_plan(d, 4096, 4096, 4100, None, 4100, 0, None, 4096, 0, None, 4096, 0, 1)
    assert s == S.OK and plan.kernel == 1                       # K not a multiple of 32: staged kernel
    # overlap is measured in bytes of the real element size
    assert P.prism_gemm(d, 64, 64, 64, FAKE_A, 64, FAKE_B, 64, FAKE_A + 64 * 64 * 4 - 4, 64, None) == S.INVALID_ARG
    s, _ = P.prism_gemm_plan(d, 64, 64, 64, FAKE_A, 64, 0, FAKE_B, 64, 0, FAKE_A + 64 * 64 * 4, 64, 0, 1)
    assert s == S.OK


def test_scan_host_validation():
    s, b = P.prism_scan_workspace_size(0)
    assert (s, b) == (S.OK, 0)
    s, b = P.prism_scan_workspace_size(1)
    assert (s, b) == (S.OK, 64 + 8)
    s, b = P.prism_scan_workspace_size(16384 * 10 + 1)
    assert (s, b) == (S.OK, 64 + 8 * 11)
    assert P.prism_scan_workspace_size(-1)[0] == S.INVALID_ARG
    assert P.prism_scan_workspace_size(1 << 43)[0] == S.INVALID_ARG
    IN, OUT, WS = FAKE, FAKE + (1 << 32), FAKE + (2 << 32)
    assert P.prism_scan_u32(None, None, 0, None, 0, None) == S.OK              # nothing to do
    assert P.prism_scan_u32(None, OUT, 100, WS, 1 << 20, None) == S.INVALID_ARG
    assert P.prism_scan_u32(IN, OUT, -5, WS, 1 << 20, None) == S.INVALID_ARG
    assert P.prism_scan_u32(IN + 2, OUT, 100, WS, 1 << 20, None) == S.INVALID_ARG     # not 4-byte aligned
    assert P.prism_scan_u32(IN, IN + 40, 100, WS, 1 << 20, None) == S.INVALID_ARG     # partial overlap
    assert P.prism_scan_u32(IN, OUT, 100, None, 0, None) == S.WORKSPACE
    assert P.prism_scan_u32(IN, OUT, 100, WS, 71, None) == S.WORKSPACE
    assert P.prism_scan_u32(IN, OUT, 100, WS + 4, 1 << 20, None) == S.INVALID_ARG     # workspace alignment
    assert P.prism_scan_u32(IN, OUT, 100, IN + 64, 1 << 20, None) == S.INVALID_ARG    # workspace inside the data
    assert P.prism_scan_check(None, None) == S.INVALID_ARG
    # the entry point with the built-in scratch: argument errors come before anything touches a GPU
    assert P.prism_scan_u32_static(IN, OUT, (1 << 30) + 1, None, None) == S.WORKSPACE   # more than the scratch holds
    assert P.prism_scan_u32_static(IN, OUT, -1, None, None) == S.INVALID_ARG
    assert P.prism_scan_u32_static(None, None, 0, None, None) == S.OK
    assert P.prism_scan_u32_static(None, OUT, 8, None, None) == S.INVALID_ARG
    assert P.prism_scan_u32_static(IN, IN + 40, 100, None, None) == S.INVALID_ARG       # partial overlap
    assert P.prism_scan_u32_static(IN, OUT, 100, IN + 2, None) == S.INVALID_ARG         # flag not 4-byte aligned
    assert P.prism_scan_u32_static(IN, OUT, 100, IN + 8, None) == S.INVALID_ARG         # flag inside the data


def test_persistent_kernel_needs_an_even_number_of_k_steps():
    d = P.make_desc()
    even = _plan(d, 512, 512, 512, batch=256)
    odd = _plan(d, 512, 512, 448, batch=256)           # 7 K steps
    assert even.kernel == 3 and odd.kernel == 2 and odd.workgroups == 1024


