"""Pins for the oracle's bf16 helpers: an independent library conversion (torch CPU) and exact
rational arithmetic."""
from fractions import Fraction

import numpy as np
import torch

import oracle


def _all_finite_bf16():
    b = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    f = oracle.bits_to_f32(b)
    return b[np.isfinite(f)]


def test_bits_roundtrip_all_patterns():
    b = _all_finite_bf16()
    assert np.array_equal(oracle.f32_to_bits(oracle.bits_to_f32(b)), b)
    assert np.array_equal(oracle.f64_to_bits(oracle.bits_to_f64(b)), b)


def test_widening_matches_torch():
    b = _all_finite_bf16()
    t = torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t.view(np.uint32), oracle.bits_to_f32(b).view(np.uint32))


def test_f32_rne_matches_torch():
    rng = np.random.default_rng(1)
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(3.0),
        (rng.standard_normal(50000) * 1e-40).astype(np.float32),          # subnormals
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, -3.3895314e38, 3.4e38], np.float32),
    ])
    ours = oracle.f32_to_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)


def _exact_rne_bf16(x):
    """Round a python float to bf16 with exact rational arithmetic (finite, normal-range results)."""
    if x == 0:
        return 0.0
    fr = Fraction(x)
    s = -1 if fr < 0 else 1
    fr = abs(fr)
    e = 0
    while fr >= 2:
        fr /= 2
        e += 1
    while fr < 1:
        fr *= 2
        e -= 1
    scaled = fr * 128                      # 7 fraction bits
    lo = scaled.numerator // scaled.denominator
    rem = scaled - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return s * float(Fraction(lo, 128) * Fraction(2) ** e)


def test_f64_single_rounding_against_rationals():
    rng = np.random.default_rng(2)
    xs = list(rng.standard_normal(3000) * 10.0)
    # values engineered to sit a hair above / below / exactly on a bf16 rounding midpoint, where
    # rounding through float32 first would go wrong
    for base in (1.0, 1.0078125, 3.5, 100.0):
        ulp = np.spacing(np.float32(base)).astype(np.float64) * 65536.0   # bf16 ulp
        mid = base + ulp / 2
        xs += [mid, mid * (1 + 2e-16), mid * (1 - 2e-16), mid + 1e-12, mid - 1e-12, -mid, -(mid + 1e-12)]
    xs = np.array(xs, dtype=np.float64)
    got = oracle.bits_to_f64(oracle.f64_to_bits(xs))
    want = np.array([_exact_rne_bf16(float(v)) for v in xs])
    assert np.array_equal(got, want)


def test_f64_overflow_and_sign():
    b = oracle.f64_to_bits(np.array([1e300, -1e300, 0.0, -0.0]))
    assert list(b) == [0x7F80, 0xFF80, 0x0000, 0x8000]
