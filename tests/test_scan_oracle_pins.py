"""Pins for the prefix-scan oracle: closed forms, brute force with Python integers,
numpy's 64-bit cumulative sum reduced modulo 2^32, and invariants.  No expected value
comes from the oracle itself or from the GPU path."""
import numpy as np
import pytest

from oracle import inclusive_scan_u32_ref
from workloads import scan_input_u32

MOD = 1 << 32


def test_all_ones_counts_positions():
    n = 100_003
    assert (inclusive_scan_u32_ref(np.ones(n, np.uint32)) == np.arange(1, n + 1, dtype=np.uint32)).all()


def test_iota_gives_triangular_numbers_with_wraparound():
    n = 200_000                                   # n(n+1)/2 exceeds 2^32 from i = 92682 on
    got = inclusive_scan_u32_ref(np.arange(n, dtype=np.uint32))
    for i in (0, 1, 2, 1000, 92_681, 92_682, 150_000, n - 1):
        assert int(got[i]) == (i * (i + 1) // 2) % MOD
    assert any((i * (i + 1) // 2) >= MOD for i in (92_682, n - 1))


def test_all_max_values_wrap():
    n = 5000
    got = inclusive_scan_u32_ref(np.full(n, 0xFFFFFFFF, np.uint32))
    want = [((i + 1) * 0xFFFFFFFF) % MOD for i in range(n)]
    assert got.tolist() == want


@pytest.mark.parametrize("n", [0, 1, 2, 3, 63, 64, 65, 257])
def test_brute_force_python_integers(n):
    x = scan_input_u32(7, n)
    got = inclusive_scan_u32_ref(x)
    assert got.shape == (n,)
    xs = [int(v) for v in x]
    for i in range(n):
        assert int(got[i]) == sum(xs[: i + 1]) % MOD   # includes position i itself


def test_against_numpy_uint64_cumsum():
    x = scan_input_u32(8, 3_000_001)
    want = (np.cumsum(x.astype(np.uint64)) % MOD).astype(np.uint32)   # 3e6 * 2^32 < 2^64: no overflow
    assert (inclusive_scan_u32_ref(x) == want).all()


def test_difference_invariant_and_single_spike():
    x = scan_input_u32(9, 70_000)
    y = inclusive_scan_u32_ref(x)
    assert y[0] == x[0]
    assert ((y[1:] - y[:-1]) == x[1:]).all()        # uint32 subtraction wraps the same way
    z = np.zeros(1000, np.uint32)
    z[417] = 12345
    got = inclusive_scan_u32_ref(z)
    assert (got[:417] == 0).all() and (got[417:] == 12345).all()
