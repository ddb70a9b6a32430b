"""bfloat16 grid helpers for the oracle (test infrastructure only).

bfloat16 = 1 sign bit, 8 exponent bits (bias 127, same as IEEE binary32), 7 explicit
fraction bits.  `round_to_bf16` rounds an fp64 array directly onto that grid with
round-to-nearest, ties-to-even (no intermediate binary32 step, so no double rounding).
"""
import numpy as np

_MIN_NORMAL_EXP = -126          # smallest normal binade of binary32 / bfloat16
_SIG_BITS = 8                   # 1 implicit + 7 explicit significand bits
_MAX_FINITE = (2.0 - 2.0 ** -7) * 2.0 ** 127


def round_to_bf16(x):
    """Nearest bfloat16 value (ties to even) of every element of fp64 array `x`, as fp64."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m * 2**e, 0.5 <= |m| < 1
    # value of one unit in the last place for the binade of x (subnormals share one ulp)
    ulp_exp = np.maximum(e - _SIG_BITS, _MIN_NORMAL_EXP + 1 - _SIG_BITS)
    q = np.rint(np.ldexp(x, -ulp_exp))       # np.rint rounds half to even
    y = np.ldexp(q, ulp_exp)
    with np.errstate(invalid="ignore"):
        y = np.where(np.abs(y) > _MAX_FINITE, np.copysign(np.inf, x), y)
    return np.where(np.isfinite(x), y, x)


def bf16_bits_to_f64(bits):
    """uint16 bfloat16 bit patterns -> exact fp64 values."""
    bits = np.asarray(bits, dtype=np.uint16)
    u32 = bits.astype(np.uint32) << np.uint32(16)
    with np.errstate(invalid="ignore"):          # signalling-NaN patterns
        return u32.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x):
    """fp64 -> uint16 bit pattern of the nearest bfloat16 (ties to even)."""
    y = round_to_bf16(x).astype(np.float32)      # exact: y is on the bf16 grid
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
