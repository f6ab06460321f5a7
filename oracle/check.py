"""Acceptance test of a GPU result against the oracle -- test infrastructure.

For every entry the accumulated fp32 value must satisfy
    |y - ref| <= 4 * K * 2^-24 * mag + 1e-6 .
When the output is stored in a narrower format (bf16 / fp16) the bound applies
to the fp32 value *before* the final conversion: the stored value C is
accepted iff some y inside the bound rounds (to nearest, ties to even) to C.
Rounding is monotone, so that is   rne(ref - bound) <= C <= rne(ref + bound).
"""
from __future__ import annotations

import numpy as np

from .reference import decode_bits

# format -> (significand bits incl. hidden one, minimum normal exponent, largest finite)
_FORMATS = {
    "bf16": (8, -126, (2.0 - 2.0 ** -7) * 2.0 ** 127),
    "f16": (11, -14, 65504.0),
    "f32": (24, -126, (2.0 - 2.0 ** -23) * 2.0 ** 127),
}


def rne_to_format(x: np.ndarray, fmt: str) -> np.ndarray:
    """Round float64 values to the nearest representable value of `fmt`
    (ties to even), returned as float64.  Written from the definition:
    the spacing of the format at |x| is 2^(e - p + 1) with e = floor(log2|x|)
    clamped to the minimum exponent; round x / spacing to the nearest integer.
    """
    p, emin, fmax = _FORMATS[fmt]
    x = np.asarray(x, dtype=np.float64)
    _, ex = np.frexp(x)                      # x = m * 2^ex, 0.5 <= |m| < 1
    e = np.maximum(ex.astype(np.int64) - 1, emin)
    spacing = np.ldexp(1.0, (e - p + 1).astype(np.int64))
    y = np.rint(x / spacing) * spacing       # np.rint rounds half to even
    y = np.where(np.abs(y) > fmax, np.copysign(np.inf, y), y)
    return np.where(np.isfinite(x), y, x)


def acceptance_bound(mag: np.ndarray, K: int) -> np.ndarray:
    return 4.0 * K * 2.0 ** -24 * np.asarray(mag, dtype=np.float64) + 1e-6


def decode_output(c: np.ndarray, c_dtype: str) -> np.ndarray:
    """Stored output -> float64.  bf16/f16 are passed as uint16 bit patterns."""
    if c_dtype == "f32":
        return np.asarray(c, dtype=np.float32).astype(np.float64)
    return decode_bits(np.asarray(c).view(np.uint16), c_dtype)


def check_against_oracle(c: np.ndarray, ref: np.ndarray, mag: np.ndarray,
                         K: int, c_dtype: str) -> dict:
    """c: decoded GPU output (float64), same shape as ref / mag."""
    c = np.asarray(c, dtype=np.float64)
    bound = acceptance_bound(mag, K)
    if c_dtype == "f32":
        lo, hi = ref - bound, ref + bound
    else:
        lo = rne_to_format(ref - bound, c_dtype)
        hi = rne_to_format(ref + bound, c_dtype)
    good = (c >= lo) & (c <= hi)
    bad = ~good
    err = np.abs(c - ref)
    ratio = err / bound
    worst = int(np.argmax(ratio)) if ratio.size else -1
    return {
        "ok": bool(good.all()),
        "n_bad": int(bad.sum()),
        "n": int(c.size),
        "max_err_over_bound": float(ratio.max()) if ratio.size else 0.0,
        "max_abs_err": float(err.max()) if err.size else 0.0,
        "worst_index": worst,
        "first_bad": (tuple(int(v) for v in np.argwhere(bad)[0]) if bad.any() else None),
    }
