"""Oracle for the 8-bit key/value cache variant: the OCP "FP8 E4M3" number format.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper does not describe a cache; an 8-bit cache is a bandwidth variant of the rollout path
whose numerical contract is stated here: every key (after QK-norm and RoPE) and every value is
stored as the E4M3 number nearest to it (ties to the even code, magnitudes above the largest
finite number 448 stored as +-448) and read back exactly.  Format (OCP 8-bit floating point
specification, E4M3): 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0
holds subnormals m/8 * 2^-6; there are no infinities; S.1111.111 is NaN, so the largest finite
code is S.1111.110 = 1.75 * 2^8.

Written from the format's definition: decode by the formula, encode by search for the nearest of
the 127 non-negative finite values.
"""
import numpy as np


def e4m3_decode(code):
    """Value of one code 0..255 (NaN for 0x7f / 0xff)."""
    code = int(code)
    sign = -1.0 if code & 0x80 else 1.0
    e, m = (code >> 3) & 0xF, code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return sign * (m / 8.0) * 2.0 ** -6
    return sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)


# the non-negative finite values in code order (code = index), strictly increasing
_POS = np.array([e4m3_decode(c) for c in range(0x7F)], np.float64)
E4M3_MAX = float(_POS[-1])


def e4m3_encode(x):
    """Codes (uint8) of the nearest E4M3 numbers: ties go to the even code, |x| > 448 saturates.
    NaN is not a valid input."""
    x = np.asarray(x, np.float64)
    if np.isnan(x).any():
        raise ValueError("NaN has no cache encoding")
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")          # first value >= a
    hi = np.minimum(hi, len(_POS) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - _POS[lo], _POS[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(x), code | np.uint8(0x80), code).astype(np.uint8)


def e4m3_round(x):
    """x stored in the cache and read back (float64)."""
    c = e4m3_encode(x)
    mag = _POS[(c & 0x7F).astype(np.int64)]
    return np.where(c & 0x80, -mag, mag)
