"""Pins for the fp32-operand entry of the CPU oracle (the paper's sgemm,
section 6.1).  Expected values come from exact rational arithmetic, hand-worked
numbers, closed forms, numpy's float64 matmul and the independent 16-bit entry
of the oracle; none comes from the function under test or from the GPU path.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import gemm_ref
from workloads import to_bf16_bits, small_integers, normal, uniform_pm1

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
LAYOUTS = list(itertools.product(["row", "col"], ["row", "col"]))


def _store(x, layout):
    return np.ascontiguousarray(x if layout == "row" else x.T)


def _ref(a, b, la="row", lb="row", **kw):
    """a: logical MxK, b: logical KxN, both exactly representable in float32."""
    M, K = a.shape
    N = b.shape[1]
    A = _store(a, la).astype(np.float32).ravel()
    B = _store(b, lb).astype(np.float32).ravel()
    assert (A.astype(np.float64) == _store(a, la).ravel()).all()
    return gemm_ref(A, B, ab_dtype="f32", M=M, N=N, K=K, layout_a=la, layout_b=lb, **kw)


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


@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_golden_hand_worked(la, lb):
    g = _read_golden("gemm_definition_2x3x2.txt")
    M, N, K = int(g["M"][0]), int(g["N"][0]), int(g["K"][0])
    a = np.array(g["A"]).reshape(M, K)
    b = np.array(g["B"]).reshape(K, N)
    ref, mag = _ref(a, b, la, lb, alpha=g["alpha"][0], beta=g["beta"][0],
                    bias=np.array(g["bias"], dtype=np.float32), c_in=np.array(g["C_in"]).reshape(M, N))
    assert (ref.ravel() == np.array(g["ref"])).all()
    assert (mag.ravel() == np.array(g["mag"])).all()


@pytest.mark.parametrize("la,lb", LAYOUTS)
def test_exact_rational_arithmetic(la, lb):
    """Full-precision float32 values (not representable in 16 bits): the exact
    result from Python fractions, within double rounding of the k sum."""
    M, N, K = 5, 4, 23
    a = normal(31, 0, M * K).astype(np.float32).reshape(M, K)
    b = (uniform_pm1(31, 1, K * N) * 3.0).astype(np.float32).reshape(K, N)
    bias = normal(31, 2, N).astype(np.float32)
    c0 = normal(31, 3, M * N).astype(np.float64).reshape(M, N)
    alpha, beta = -1.25, 0.5
    ref, mag = _ref(a.astype(np.float64), b.astype(np.float64), la, lb, alpha=alpha, beta=beta, bias=bias, c_in=c0)
    for i in range(M):
        for j in range(N):
            s = sum(Fraction(float(a[i, k])) * Fraction(float(b[k, j])) for k in range(K))
            m = sum(abs(Fraction(float(a[i, k])) * Fraction(float(b[k, j]))) for k in range(K))
            want = Fraction(alpha) * s + Fraction(float(bias[j])) + Fraction(beta) * Fraction(float(c0[i, j]))
            wmag = abs(Fraction(alpha)) * m + abs(Fraction(float(bias[j]))) + abs(Fraction(beta) * Fraction(float(c0[i, j])))
            assert abs(Fraction(float(ref[i, j])) - want) <= Fraction(1, 2 ** 48) * wmag
            assert abs(Fraction(float(mag[i, j])) - wmag) <= Fraction(1, 2 ** 48) * wmag


def test_identity_permutation_and_ones():
    n = 129
    a = normal(32, 0, 40 * n).astype(np.float32).astype(np.float64).reshape(40, n)
    for la, lb in LAYOUTS:
        ref, mag = _ref(a, np.eye(n), la, lb)
        assert (ref == a).all() and (mag == np.abs(a)).all()
        ref, _ = _ref(np.eye(n), a.T.copy(), la, lb)
        assert (ref == a.T).all()
    rng = np.random.default_rng(7)
    pi = rng.permutation(n)
    P = np.zeros((n, n))
    P[pi, np.arange(n)] = 1.0
    ref, _ = _ref(a, P)
    assert (ref == a[:, pi]).all()
    ref, mag = _ref(np.ones((7, 4096)), np.ones((4096, 3)))
    assert (ref == 4096).all() and (mag == 4096).all()


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (1, 2, 2), (2, 1, 2), (2, 2, 1), (2, 2, 2)])
def test_exhaustive_tiny(M, N, K):
    """Every matrix pair over {-1, 0, 1} against Python integers."""
    vals = (-1.0, 0.0, 1.0)
    for ea in itertools.product(vals, repeat=M * K):
        a = np.array(ea).reshape(M, K)
        for eb in itertools.product(vals, repeat=K * N):
            b = np.array(eb).reshape(K, N)
            ref, mag = _ref(a, b)
            for i in range(M):
                for j in range(N):
                    assert ref[i, j] == sum(int(a[i, k]) * int(b[k, j]) for k in range(K))
                    assert mag[i, j] == sum(abs(int(a[i, k]) * int(b[k, j])) for k in range(K))


def test_against_numpy_f64_all_layouts_with_padding():
    M, N, K = 37, 53, 129
    a = normal(33, 0, M * K).astype(np.float32).astype(np.float64).reshape(M, K)
    b = normal(33, 1, K * N).astype(np.float32).astype(np.float64).reshape(K, N)
    bias = normal(33, 2, N).astype(np.float32)
    c0 = normal(33, 3, M * N).astype(np.float64).reshape(M, N)
    want = 1.5 * (a @ b) + bias.astype(np.float64)[None, :] + 0.75 * c0
    wmag = 1.5 * (np.abs(a) @ np.abs(b)) + np.abs(bias.astype(np.float64))[None, :] + np.abs(0.75 * c0)
    for la, lb in LAYOUTS:
        ref, mag = _ref(a, b, la, lb, alpha=1.5, beta=0.75, bias=bias, c_in=c0)
        assert np.abs(ref - want).max() <= 1e-12 * wmag.max()
        assert np.abs(mag - wmag).max() <= 1e-12 * wmag.max()
    # padded leading dimensions, row-major A (lda 140) and row-major B (ldb 60)
    Ap = np.full((M, 140), 7.0, dtype=np.float32)
    Ap[:, :K] = a
    Bp = np.full((K, 60), -7.0, dtype=np.float32)
    Bp[:, :N] = b
    ref, _ = gemm_ref(Ap.ravel(), Bp.ravel(), ab_dtype="f32", M=M, N=N, K=K, layout_a="row", layout_b="row",
                      lda=140, ldb=60)
    assert np.abs(ref - a @ b).max() <= 1e-12 * (np.abs(a) @ np.abs(b)).max()
    rows = [36, 0, 5, 5]
    sub, _ = _ref(a, b, rows=rows)
    full, _ = _ref(a, b)
    assert (sub == full[rows]).all()


def test_agrees_with_the_16_bit_entry_on_shared_values():
    """Values representable in bf16 go through both entries of the oracle (separate
    decoders and loops): results must be identical."""
    M, N, K = 19, 23, 77
    a = small_integers(34, 0, M * K, -8, 8).reshape(M, K).astype(np.float64) / 4.0
    b = small_integers(34, 1, K * N, -8, 8).reshape(K, N).astype(np.float64) / 8.0
    r32, m32 = _ref(a, b, "row", "col", alpha=0.5)
    r16, m16 = gemm_ref(to_bf16_bits(a.ravel()), to_bf16_bits(np.ascontiguousarray(b.T).ravel()), ab_dtype="bf16",
                        M=M, N=N, K=K, layout_a="row", layout_b="col", alpha=0.5)
    assert (r32 == r16).all() and (m32 == m16).all()


def test_k_zero_and_storage_type_is_checked():
    bias = np.array([1.5, -2.0], dtype=np.float32)
    r, m = gemm_ref(np.zeros(0, np.float32), np.zeros(0, np.float32), ab_dtype="f32", M=3, N=2, K=0, bias=bias)
    assert (r == bias.astype(np.float64)[None, :]).all() and (m == np.abs(r)).all()
    with pytest.raises(AssertionError):
        gemm_ref(np.zeros(4, np.uint16), np.zeros(4, np.uint16), ab_dtype="f32", M=2, N=2, K=2)
