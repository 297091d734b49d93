"""bf16 <-> fp64 helpers for the oracle (bit patterns as numpy.uint16)."""

import numpy as np


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of each bf16 bit pattern as float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 to the nearest bf16 value (ties to even); result stays float64.

    bf16 keeps 8 significant bits; below 2**-126 the spacing is fixed at 2**-133.
    """
    x = np.asarray(x, dtype=np.float64)
    if not np.all(np.isfinite(x)):
        raise ValueError("non-finite value")
    m, e = np.frexp(x)  # x = m * 2**e, 0.5 <= |m| < 1
    normal = e > -126
    qn = np.ldexp(np.rint(m * 256.0) / 256.0, e)
    qs = np.rint(x * 2.0**133) * 2.0**-133
    out = np.where(normal, qn, qs)
    if np.any(np.abs(out) > 3.3895313892515355e38):
        raise ValueError("overflows bf16")
    return out


def f64_to_bits(x: np.ndarray) -> np.ndarray:
    """Round to bf16 and return the bit pattern."""
    y = round_to_bf16(x).astype(np.float32)  # exact: y has <= 8 significant bits
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
