"""Counter-based random inputs: every element is a pure function of
(seed, tensor_id, linear index), so any slice can be regenerated on its own.

The paper initialises its benchmark operands from a random number generator
(evaluation set-up, section 6); these generators are the stand-in.  Nothing in
this file multiplies matrices.
"""
from __future__ import annotations

import numpy as np

_U64 = np.uint64
_CHUNK = 1 << 22  # elements drawn per slab, bounds temporary memory


def _mix64(x: np.ndarray) -> np.ndarray:
    """SplitMix64 output function (Steele, Lea, Flood 2014) on uint64 arrays."""
    x = (x + _U64(0x9E3779B97F4A7C15))
    x = (x ^ (x >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
    x = (x ^ (x >> _U64(27))) * _U64(0x94D049BB133111EB)
    return x ^ (x >> _U64(31))


def _hash(seed: int, tensor_id: int, start: int, count: int, stream: int) -> np.ndarray:
    idx = np.arange(start, start + count, dtype=_U64)
    key = _mix64(np.array([(seed << 8) ^ (tensor_id << 4) ^ stream], dtype=_U64))[0]
    with np.errstate(over="ignore"):
        return _mix64(idx ^ key)


def _u01(seed, tensor_id, start, count, stream) -> np.ndarray:
    """24-bit uniform in [0, 1) as float64."""
    h = _hash(seed, tensor_id, start, count, stream)
    return (h >> _U64(40)).astype(np.float64) * (1.0 / (1 << 24))


def _slabs(n: int):
    for s in range(0, n, _CHUNK):
        yield s, min(_CHUNK, n - s)


def uniform_pm1(seed: int, tensor_id: int, n: int) -> np.ndarray:
    """n float32 values uniform in [-1, 1)."""
    out = np.empty(n, dtype=np.float32)
    for s, c in _slabs(n):
        out[s:s + c] = (2.0 * _u01(seed, tensor_id, s, c, 0) - 1.0).astype(np.float32)
    return out


def normal(seed: int, tensor_id: int, n: int, sigma: float = 1.0) -> np.ndarray:
    """n float32 values ~ N(0, sigma^2) by the Box-Muller transform."""
    out = np.empty(n, dtype=np.float32)
    for s, c in _slabs(n):
        u1 = _u01(seed, tensor_id, s, c, 1)
        u2 = _u01(seed, tensor_id, s, c, 2)
        r = np.sqrt(-2.0 * np.log(1.0 - u1))          # 1-u1 in (0, 1]
        out[s:s + c] = (sigma * r * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    return out


def small_integers(seed: int, tensor_id: int, n: int, lo: int = -8, hi: int = 8) -> np.ndarray:
    """n float32 values that are integers in [lo, hi] (exact in bf16 and fp16)."""
    span = _U64(hi - lo + 1)
    out = np.empty(n, dtype=np.float32)
    for s, c in _slabs(n):
        h = _hash(seed, tensor_id, s, c, 3)
        out[s:s + c] = ((h >> _U64(16)) % span).astype(np.float32) + np.float32(lo)
    return out


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even. Finite input only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def to_f16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> IEEE half bit patterns (uint16), round to nearest even."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def encode(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return to_bf16_bits(x)
    if dtype == "f16":
        return to_f16_bits(x)
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32)
    raise ValueError(dtype)


def scan_input_u32(seed: int, n: int) -> np.ndarray:
    """n uint32 values covering the full 32-bit range (prefix sums wrap often)."""
    out = np.empty(n, dtype=np.uint32)
    for s, c in _slabs(n):
        out[s:s + c] = (_hash(seed, 5, s, c, 0) >> _U64(32)).astype(np.uint32)
    return out
