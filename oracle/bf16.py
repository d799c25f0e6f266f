"""bfloat16 <-> float64 conversion for the oracle (test infrastructure only).

bfloat16 = 1 sign bit, 8 exponent bits, 7 stored mantissa bits, i.e. the upper
half of an IEEE float32.  Tensors are carried as numpy uint16 bit patterns.

Rounding is done straight from float64 to the 8-bit significand (round to
nearest, ties to even), not through float32, so there is no double rounding.
"""
from __future__ import annotations

import numpy as np


def widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float64 (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    f32 = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return f32.astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float64 -> bf16 bit patterns, round-to-nearest-even on the 8-bit significand.

    x = m * 2**e with 0.5 <= |m| < 1; a bf16 normal keeps 8 significant bits, so
    the representable neighbours are multiples of 2**(e-8).  Below the smallest
    normal (2**-126) the spacing is fixed at 2**-133 (subnormals).  np.rint
    rounds halves to even.  Values whose rounded magnitude exceeds the largest
    finite bf16 become infinity; NaN stays NaN.
    """
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    e = np.maximum(e, -125)                       # subnormal range: fixed quantum 2**-133
    quantum = np.ldexp(1.0, e - 8)
    with np.errstate(invalid="ignore"):
        y = np.rint(x / quantum) * quantum
    y = np.where(np.isfinite(x), y, x)
    max_bf16 = float.fromhex("0x1.fep127")
    y = np.where(np.abs(y) > max_bf16, np.copysign(np.inf, y), y)
    f32 = y.astype(np.float32)                    # exact: y has <= 8 significant bits
    return (f32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
