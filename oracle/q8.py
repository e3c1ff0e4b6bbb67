"""8-bit storage of the condensed representatives — TEST INFRASTRUCTURE ONLY (same rule as the rest of
this package: only the tests, ``smoke()`` and the CPU-baseline leg of ``bench.py`` may import it).

The paper leaves formats below 16 bits unexplored (limitations section), so the format is this build's own
reading, written out here step by step in float64:

* codes are OCP FP8 E4M3 ("e4m3fn"): 1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent field 0 holds the
  subnormals m/8 * 2^-6, exponent 15 with mantissa 7 is NaN, there are no infinities, the largest finite
  value is 1.75 * 2^8 = 448;
* every representative row carries one scale per component (pooled part, selected part), a power of two
  chosen so that the row's largest magnitude lands in (224, 448] (scale 1 for an all-zero row);
* a value x is stored as the code nearest to x / scale, ties to the code with the even mantissa, the
  sign bit being the sign of x (also when the magnitude rounds to zero);
* the stored value is decode(code) * scale.
Since the scale is a power of two, x / scale is exact and the only rounding is the one to the code.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode_table() -> np.ndarray:
    """Value of each of the 256 codes (NaN for the two NaN codes), from the format's definition."""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e, m = (code >> 3) & 0xF, code & 0x7
        if e == 15 and m == 7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * (m / 8.0) * 2.0 ** -6
        else:
            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


_POS = e4m3_decode_table()[:0x7F]          # the 127 non-negative finite values, ascending with the code


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest code for every element of x (float64): ties to the even code, magnitudes beyond 448 saturate."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")            # first code whose value is >= a
    hi = np.minimum(hi, len(_POS) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - _POS[lo], _POS[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return code | (np.signbit(x).astype(np.uint8) << 7)


def row_scale(amax: np.ndarray) -> np.ndarray:
    """Power of two s with amax / s in (224, 448]; 1 where amax is 0."""
    amax = np.asarray(amax, dtype=np.float64)
    f, e = np.frexp(amax)                                  # amax = f * 2^e, f in [0.5, 1)
    s = np.where(f <= 0.875, np.ldexp(1.0, e - 9), np.ldexp(1.0, e - 8))      # 448 = 0.875 * 2^9
    return np.where(amax == 0.0, 1.0, s)


def quantize_rows(x: np.ndarray):
    """x [..., d] float64 -> (codes uint8 [..., d], scale float64 [...])."""
    x = np.asarray(x, dtype=np.float64)
    s = row_scale(np.abs(x).max(axis=-1))
    return e4m3_encode(x / s[..., None]), s


def dequantize_rows(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    return e4m3_decode_table()[codes] * np.asarray(scale, dtype=np.float64)[..., None]
