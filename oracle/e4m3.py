"""OCP FP8 E4M3 ("e4m3fn") codec in float64 NumPy -- TEST INFRASTRUCTURE ONLY.

Part of the CPU oracle.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
import it; the product path never does, and this file shares no code with the HIP kernels.

Format (fixed by the paper's constant 448 = largest finite magnitude, Sec. 3.2, "fixed scalar
1/448"): 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, the single
NaN pattern S.1111.111, subnormals m * 2^-9 for exponent field 0.  Rounding is to nearest with
ties to the even mantissa, and magnitudes above 448 saturate to 448 (the paper states no
rounding rule; this is the reading taken and recorded in the design notes).
"""
from __future__ import annotations

import numpy as np

FP8_MAX = 448.0            # M_FP8max of Eq. 4
_MIN_NORMAL_EXP = -6       # smallest normal magnitude 2^-6
_SUBNORMAL_QUANTUM = -9    # subnormals are multiples of 2^-9


def decode_table() -> np.ndarray:
    """Value of every byte code 0..255 as float64 (the two NaN codes decode to NaN)."""
    vals = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            vals[code] = np.nan
        elif e == 0:
            vals[code] = sign * m * 2.0 ** _SUBNORMAL_QUANTUM
        else:
            vals[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return vals


_DECODE = decode_table()
_POS = _DECODE[:0x7F].copy()                 # 127 non-negative finite values, ascending
_MID = 0.5 * (_POS[:-1] + _POS[1:])          # 126 rounding midpoints (exact in float64)


def decode(codes: np.ndarray) -> np.ndarray:
    """Byte codes -> float64 values."""
    return _DECODE[np.asarray(codes, dtype=np.uint8)]


def encode_scaled(x: np.ndarray, s: float) -> np.ndarray:
    """Codes of round-to-nearest-even(x / s), saturating, with the quotient taken exactly.

    x holds bf16 values (8 significant bits) and s a float32 value, both as float64, so each
    threshold mid*s (5 bits x 24 bits) is exact in float64 and the comparison |x| vs mid*s decides
    on which side of a rounding midpoint the exact quotient lies (Eq. 1 / Eq. 5 with the scale of
    Eq. 4: encode x/s, decode code*s).
    """
    x = np.asarray(x, dtype=np.float64)
    s = float(s)
    assert s > 0.0 and np.isfinite(s)
    a = np.abs(x)
    th = _MID * s
    k = np.searchsorted(th, a, side="left")          # number of thresholds strictly below |x|
    tie = (k < th.size) & (a == th[np.minimum(k, th.size - 1)])
    k = np.where(tie & (k % 2 == 1), k + 1, k)       # on a tie take the even code (even mantissa)
    codes = k.astype(np.uint8)
    codes = np.where(np.signbit(x), codes | np.uint8(0x80), codes).astype(np.uint8)
    return codes


def round_to_e4m3(y: np.ndarray) -> np.ndarray:
    """Nearest e4m3fn value (ties to even, saturating) of each float64 y, as float64.

    Arithmetic form: a value with binary exponent e keeps 4 significant bits, i.e. is a multiple
    of 2^(e-3); below 2^-6 the quantum stays 2^-9.  np.rint rounds halves to even.
    """
    y = np.asarray(y, dtype=np.float64)
    a = np.minimum(np.abs(y), FP8_MAX)
    _, e = np.frexp(a)                                # a = f * 2^e, f in [0.5, 1)
    q = np.maximum(e - 4, _SUBNORMAL_QUANTUM)         # quantum exponent
    r = np.ldexp(np.rint(np.ldexp(a, -q)), q)
    return np.copysign(np.minimum(r, FP8_MAX), y)


def encode(y: np.ndarray) -> np.ndarray:
    """Byte codes of round_to_e4m3(y)."""
    return encode_scaled(y, 1.0)
