"""bf16 <-> fp64 conversions of the CPU oracle (test infrastructure only).

bf16 is the upper half of an IEEE fp32: 1 sign, 8 exponent, 7 mantissa bits.
"""
import numpy as np


def bf16_bits_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16)
    return (u.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x) -> np.ndarray:
    """Round fp64 to bf16, nearest, ties to even; returns uint16 bit patterns.

    Done in one rounding: the two bf16 neighbours of x are formed and the nearer
    one (in fp64) is taken, so there is no double rounding through fp32.
    """
    x = np.asarray(x, dtype=np.float64)
    f32 = x.astype(np.float32)
    b = f32.view(np.uint32)
    toward_zero = b & np.uint32(0xFFFF0000)
    away = toward_zero + np.uint32(0x00010000)
    lo = toward_zero.view(np.float32).astype(np.float64)
    hi = away.view(np.float32).astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        d_lo = np.abs(x - lo)
        d_hi = np.abs(hi - x)
    lo_is_even = (toward_zero & np.uint32(0x00010000)) == 0
    take_lo = (d_lo < d_hi) | ((d_lo == d_hi) & lo_is_even)
    finite = np.isfinite(x)
    out = np.where(take_lo | ~finite, toward_zero, away)
    # NaN: keep a quiet NaN pattern whatever the payload was.
    out = np.where(np.isnan(x), np.uint32(0x7FC00000), out)
    return (out >> np.uint32(16)).astype(np.uint16)
