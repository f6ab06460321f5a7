"""Pins for the CPU oracle: closed forms, brute force and library special
cases that a dropped term, a wrong sign/index or a transposed operand breaks.
None of the expected values comes from the oracle itself or from the GPU path.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import gemm_ref, decode_bits
from workloads import to_bf16_bits, to_f16_bits, small_integers, uniform_pm1, normal

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ENC = {"bf16": to_bf16_bits, "f16": to_f16_bits}


def _store(x, layout):
    """logical [r, c] float array -> stored flat array for the layout."""
    return np.ascontiguousarray(x if layout == "row" else x.T)


def _ref(a, b, dtype="bf16", la="row", lb="col", **kw):
    """a: logical MxK floats (exactly representable), b: logical KxN."""
    M, K = a.shape
    N = b.shape[1]
    A = ENC[dtype](_store(a, la).ravel())
    B = ENC[dtype](_store(b, lb).ravel())
    return gemm_ref(A, B, ab_dtype=dtype, M=M, N=N, K=K, layout_a=la, layout_b=lb, **kw)


def _ints(seed, tid, r, c, lo=-8, hi=8):
    return small_integers(seed, tid, r * c, lo, hi).reshape(r, c).astype(np.float64)


LAYOUTS = list(itertools.product(["row", "col"], ["row", "col"]))


# ---- decoders: every 16-bit pattern against numpy's own interpretation -------------------

def test_decode_bf16_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = decode_bits(bits, "bf16")
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == want[~nan]).all()
    assert (np.signbit(got[~nan]) == np.signbit(want[~nan])).all()


def test_decode_f16_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = decode_bits(bits, "f16")
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == want[~nan]).all()
    assert (np.signbit(got[~nan]) == np.signbit(want[~nan])).all()


# ---- hand-worked golden instance ------------------------------------------------------

def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_golden_hand_worked(dtype, la, lb):
    g = _read_golden("gemm_definition_2x3x2.txt")
    M, N, K = int(g["M"][0]), int(g["N"][0]), int(g["K"][0])
    a = np.array(g["A"]).reshape(M, K)
    b = np.array(g["B"]).reshape(K, N)
    ref, mag = _ref(a, b, dtype, la, lb, alpha=g["alpha"][0], beta=g["beta"][0],
                    bias=np.array(g["bias"], dtype=np.float32),
                    c_in=np.array(g["C_in"]).reshape(M, N))
    assert (ref.ravel() == np.array(g["ref"])).all()
    assert (mag.ravel() == np.array(g["mag"])).all()


# ---- closed forms ----------------------------------------------------------------------

@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_identity_right_and_left(la, lb):
    n = 256
    a = uniform_pm1(11, 0, 96 * n).reshape(96, n)
    a = decode_bits(to_bf16_bits(a.ravel()), "bf16").reshape(96, n)  # representable values
    ref, mag = _ref(a, np.eye(n), "bf16", la, lb)
    assert (ref == a).all() and (mag == np.abs(a)).all()
    ref, _ = _ref(np.eye(n), a.T.copy(), "bf16", la, lb)
    assert (ref == a.T).all()


@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_permutation(la, lb):
    rng = np.random.default_rng(5)
    n, m = 257, 33
    a = _ints(12, 0, m, n)
    pi = rng.permutation(n)
    P = np.zeros((n, n))
    P[pi, np.arange(n)] = 1.0             # (A P)[:, j] = A[:, pi[j]]
    ref, _ = _ref(a, P, "bf16", la, lb)
    assert (ref == a[:, pi]).all()
    b = _ints(12, 1, n, m)
    Q = np.zeros((n, n))
    Q[np.arange(n), pi] = 1.0             # (Q B)[i, :] = B[pi[i], :]
    ref, _ = _ref(Q, b, "bf16", la, lb)
    assert (ref == b[pi, :]).all()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (3, 5, 4096), (17, 2, 1)])
def test_all_ones_gives_K(dtype, M, N, K):
    ref, mag = _ref(np.ones((M, K)), np.ones((K, N)), dtype)
    assert (ref == K).all() and (mag == K).all()


def test_rank_one():
    M = N = K = 256
    u = _ints(13, 0, M, 1, -4, 4)
    v = _ints(13, 1, 1, K, -4, 4)
    a = u @ v                               # entries in [-16, 16]: exact in bf16
    ref, mag = _ref(a, np.ones((K, N)), "bf16", "row", "row")
    assert (ref == u * v.sum()).all()
    assert (mag == np.abs(u) * np.abs(v).sum()).all()
    # K = 1: a plain outer product
    w = _ints(13, 2, 1, N)
    ref, _ = _ref(u, w, "bf16", "row", "row")
    assert (ref == u * w).all()


# ---- brute force on tiny shapes --------------------------------------------------------

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (1, 1, 2), (1, 2, 1), (2, 1, 1), (2, 1, 2),
                                   (1, 2, 2), (2, 2, 1), (2, 2, 2), (1, 1, 3), (1, 3, 2)])
def test_exhaustive_tiny(M, N, K):
    """All matrices over {-1, 0, 1} against integer arithmetic in pure Python."""
    vals = (-1, 0, 1)
    for la, lb in (("row", "col"), ("col", "row")):
        for ea in itertools.product(vals, repeat=M * K):
            a = np.array(ea, dtype=np.float64).reshape(M, K)
            for eb in itertools.product(vals, repeat=K * N):
                b = np.array(eb, dtype=np.float64).reshape(K, N)
                ref, mag = _ref(a, b, "bf16", la, lb)
                for i in range(M):
                    for j in range(N):
                        s = sum(ea[i * K + k] * eb[k * N + j] for k in range(K))
                        m = sum(abs(ea[i * K + k] * eb[k * N + j]) for k in range(K))
                        assert ref[i, j] == s and mag[i, j] == m


# ---- invariants ------------------------------------------------------------------------

def test_power_of_two_scaling_and_alpha():
    a = _ints(14, 0, 19, 40)
    b = _ints(14, 1, 40, 23)
    r1, m1 = _ref(a, b)
    r2, m2 = _ref(4.0 * a, b)
    assert (r2 == 4.0 * r1).all() and (m2 == 4.0 * m1).all()
    r3, m3 = _ref(a, b, alpha=-0.25)
    assert (r3 == -0.25 * r1).all() and (m3 == 0.25 * m1).all()


def test_transpose_identity_all_layouts():
    """(A B)^T = B^T A^T, evaluated through every storage layout."""
    a = _ints(15, 0, 21, 34)
    b = _ints(15, 1, 34, 13)
    base, _ = _ref(a, b, "bf16", "row", "col")
    for la, lb in LAYOUTS:
        r, _ = _ref(a, b, "bf16", la, lb)
        assert (r == base).all()
        rt, _ = _ref(b.T.copy(), a.T.copy(), "bf16", la, lb)
        assert (rt == base.T).all()


def test_non_square_not_symmetric_against_numpy_f64():
    """Random non-square case; numpy's float64 matmul is the library routine
    the definition reduces to (agreement to rounding, not bit-for-bit)."""
    for dtype in ("bf16", "f16"):
        for la, lb in LAYOUTS:
            M, N, K = 37, 53, 129
            a = decode_bits(ENC[dtype](normal(16, 0, M * K)), dtype).reshape(M, K)
            b = decode_bits(ENC[dtype](normal(16, 1, K * N)), dtype).reshape(K, N)
            bias = normal(16, 2, N)
            c0 = normal(16, 3, M * N).astype(np.float64).reshape(M, N)
            ref, mag = _ref(a, b, dtype, la, lb, alpha=1.5, beta=0.75, bias=bias, c_in=c0)
            want = 1.5 * (a @ b) + bias.astype(np.float64)[None, :] + 0.75 * c0
            wmag = 1.5 * (np.abs(a) @ np.abs(b)) + np.abs(bias.astype(np.float64))[None, :] \
                + np.abs(0.75 * c0)
            assert np.abs(ref - want).max() <= 1e-12 * wmag.max()
            assert np.abs(mag - wmag).max() <= 1e-12 * wmag.max()


def test_leading_dimension_padding():
    a = _ints(17, 0, 9, 12)
    b = _ints(17, 1, 12, 7)
    base, _ = _ref(a, b)
    Ap = np.full((9, 20), 99.0)
    Ap[:, :12] = a                          # row-major A with lda = 20
    Bp = np.full((7, 16), -99.0)
    Bp[:, :12] = b.T                        # col-major B with ldb = 16
    r, _ = gemm_ref(to_bf16_bits(Ap.ravel()), to_bf16_bits(Bp.ravel()), ab_dtype="bf16",
                    M=9, N=7, K=12, lda=20, ldb=16)
    assert (r == base).all()


def test_row_subset_matches_full():
    a = _ints(18, 0, 40, 31)
    b = _ints(18, 1, 31, 22)
    full, fmag = _ref(a, b)
    rows = [39, 0, 7, 7, 18]
    sub, smag = _ref(a, b, rows=rows)
    assert (sub == full[rows]).all() and (smag == fmag[rows]).all()


def test_k_zero_is_bias_broadcast_and_empty_shapes():
    bias = np.array([1.5, -2.0, 0.0], dtype=np.float32)
    r, m = gemm_ref(np.zeros(0, np.uint16), np.zeros(0, np.uint16), ab_dtype="bf16",
                    M=4, N=3, K=0, bias=bias)
    assert (r == bias.astype(np.float64)[None, :]).all() and (m == np.abs(r)).all()
    r, _ = gemm_ref(np.zeros(0, np.uint16), np.zeros(0, np.uint16), ab_dtype="bf16",
                    M=4, N=3, K=0)
    assert (r == 0).all()
    r, _ = gemm_ref(np.zeros(0, np.uint16), np.zeros(8, np.uint16), ab_dtype="bf16",
                    M=0, N=2, K=4)
    assert r.shape == (0, 2)


def test_subnormal_and_signed_zero_inputs():
    # smallest fp16 subnormal squared = 2^-48, exact in double
    a = np.array([[0x0001, 0x8001]], dtype=np.uint16)        # [+2^-24, -2^-24]
    b = np.array([[0x0001, 0x0001]], dtype=np.uint16)        # col-major 2x1
    r, m = gemm_ref(a, b, ab_dtype="f16", M=1, N=1, K=2)
    assert r[0, 0] == 0.0 and m[0, 0] == 2.0 ** -47
