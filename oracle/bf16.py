"""bf16 helpers for the CPU oracle (test infrastructure only; shares nothing with the HIP path).

bf16 is carried as uint16 bit patterns.  Rounding is round-to-nearest-even (RNE) everywhere,
the rounding the paper's bf16 training setup implies (Section 4 trains in bf16; it names no
other rounding mode).
"""
import numpy as np


def bits_to_f32(bits):
    """Exact widening of bf16 bit patterns to float32."""
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bits_to_f64(bits):
    """Exact widening of bf16 bit patterns to float64."""
    return bits_to_f32(bits).astype(np.float64)


def f32_to_bits(x):
    """RNE float32 -> bf16 bit pattern (NaN -> quiet NaN with the sign kept)."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u.astype(np.uint64) + np.uint64(0x7FFF) + lsb.astype(np.uint64)) >> np.uint64(16)).astype(np.uint16)
    nan = np.isnan(f)
    if np.any(nan):
        r = np.where(nan, ((u >> np.uint32(16)).astype(np.uint16) | np.uint16(0x7FC0)), r)
    return r.astype(np.uint16)


def f64_to_bits(x):
    """Correctly rounded (single RNE) float64 -> bf16 bit pattern.

    Goes through float32 with round-to-odd, which makes the second rounding (to the 8-bit
    bf16 significand) see exactly the information a direct rounding would.
    """
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        f = x.astype(np.float32)
        back = f.astype(np.float64)
        inexact = back != x
        too_big = np.abs(back) > np.abs(x)
        trunc = np.where(too_big, np.nextafter(f, np.float32(0.0)), f).astype(np.float32)
    u = np.ascontiguousarray(trunc).view(np.uint32) | (inexact & ~np.isnan(x)).astype(np.uint32)
    return f32_to_bits(u.view(np.float32))
