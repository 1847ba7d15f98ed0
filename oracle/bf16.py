"""bfloat16 storage helpers for the oracle (bit patterns held in uint16).

bf16 = the top 16 bits of an IEEE-754 binary32: 1 sign, 8 exponent, 7 mantissa
bits.  Widening is exact.  Narrowing rounds to nearest, ties to even, taken
directly from the float64 value (no intermediate binary32 rounding, which
could double-round).
"""
import numpy as np


def to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def from_f64(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bf16 (ties to even); finite inputs."""
    x = np.asarray(x, dtype=np.float64)
    # candidate toward zero: truncate the binary32 that is itself truncated
    # toward zero from x (so no rounding has happened yet)
    f32 = x.astype(np.float32)
    # fix up binary32 conversions that rounded away from zero
    away = np.abs(f32.astype(np.float64)) > np.abs(x)
    f32 = np.where(away, np.nextafter(f32, np.float32(0)), f32).astype(np.float32)
    u = f32.view(np.uint32)
    lo = u & np.uint32(0xFFFF0000)                    # bf16 toward zero
    hi = lo + np.uint32(0x00010000)                   # next bf16 away from zero
    lo_v = lo.view(np.float32).astype(np.float64)
    hi_v = hi.view(np.float32).astype(np.float64)
    d_lo = np.abs(x - lo_v)
    d_hi = np.abs(hi_v - x)
    lo_even = ((lo >> np.uint32(16)) & np.uint32(1)) == 0
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ~lo_even)
    out = np.where(pick_hi, hi, lo)
    return (out >> np.uint32(16)).astype(np.uint16)
