"""Pins for the oracle's bf16 conversions: exact rational decoding, exhaustive
round trip, exact midpoints (ties to even), and a double-rounding trap."""
import math
import random
from fractions import Fraction

import numpy as np

from exact import bf16_to_fraction, fraction_to_bf16


def _finite_patterns():
    return [b for b in range(1 << 16) if ((b >> 7) & 0xFF) != 0xFF]


def test_decode_matches_exact_rational(oracle):
    pats = np.array(_finite_patterns(), np.uint16)
    got = oracle.bf16_to_f64(pats)
    for b, g in zip(pats.tolist(), got.tolist()):
        assert Fraction(g) == bf16_to_fraction(b), hex(b)


def test_round_trip_all_patterns(oracle):
    pats = np.array(_finite_patterns(), np.uint16)
    back = oracle.f64_to_bf16(oracle.bf16_to_f64(pats))
    # -0.0 keeps its sign, every finite value maps to itself
    assert np.array_equal(back, pats)


def test_inf_nan_overflow(oracle):
    f = oracle.f64_to_bf16
    assert f(np.array([np.inf, -np.inf]))[0] == 0x7F80 and f(np.array([-np.inf]))[0] == 0xFF80
    assert (f(np.array([np.nan]))[0] & 0x7FFF) > 0x7F80
    big = float(bf16_to_fraction(0x7F7F))          # largest finite bf16
    half_ulp = math.ldexp(1.0, 127 - 8)
    assert f(np.array([big + half_ulp * 0.999]))[0] == 0x7F7F
    assert f(np.array([big + half_ulp]))[0] == 0x7F80   # tie: 0x7F7F is odd -> rounds up to inf
    assert f(np.array([1e300]))[0] == 0x7F80 and f(np.array([-1e300]))[0] == 0xFF80


def test_midpoints_tie_to_even_and_neighbours(oracle):
    lo = np.arange(0x0000, 0x7F7F, dtype=np.uint16)      # all adjacent finite positive pairs
    hi = lo + 1
    a = oracle.bf16_to_f64(lo)
    b = oracle.bf16_to_f64(hi)
    mid = (a + b) / 2                                    # exact: one extra bit
    want = np.where(lo & 1, hi, lo)                      # even mantissa wins
    assert np.array_equal(oracle.f64_to_bf16(mid), want)
    assert np.array_equal(oracle.f64_to_bf16(-mid), want | 0x8000)
    up = np.nextafter(mid, np.inf)
    dn = np.nextafter(mid, -np.inf)
    assert np.array_equal(oracle.f64_to_bf16(up), hi)
    assert np.array_equal(oracle.f64_to_bf16(dn), lo)


def test_no_double_rounding_through_fp32(oracle):
    # 1 + 2^-8 is the midpoint of bf16 1.0 and 1.0078125.  Adding 2^-30 puts the
    # value above the midpoint; rounding to fp32 first would land ON the midpoint
    # and the tie would go down to the even 0x3F80.
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert np.float32(x) == np.float32(1.0 + 2.0 ** -8)
    assert oracle.f64_to_bf16(np.array([x]))[0] == 0x3F81
    assert oracle.f64_to_bf16(np.array([-x]))[0] == 0xBF81


def test_random_doubles_against_exact_rational(oracle):
    rnd = random.Random(1234)
    xs = []
    for _ in range(4000):
        e = rnd.choice([rnd.randint(-140, -120), rnd.randint(-20, 20), rnd.randint(120, 127)])
        xs.append(math.ldexp(rnd.uniform(-2, 2), e))
    got = oracle.f64_to_bf16(np.array(xs))
    for x, g in zip(xs, got.tolist()):
        assert g == fraction_to_bf16(Fraction(x)), x


def test_ulp_diff_hand_cases(oracle):
    a = np.array([0x3F80, 0x0000, 0x0001, 0x3F80, 0xBF80, 0x4000], np.uint16)
    b = np.array([0x3F81, 0x8000, 0x8001, 0x3F80, 0xBF7E, 0x3FFF], np.uint16)
    # 1 step up; +0 vs -0 coincide; smallest subnormals of either sign are 2 apart;
    # equal; two steps toward zero on the negative side; one step across a binade
    mx, nd = oracle.ulp_diff(a, b)
    assert (mx, nd) == (2, 4)
    assert oracle.ulp_diff(a[:1], b[:1]) == (1, 1)
    assert oracle.ulp_diff(a[1:2], b[1:2]) == (0, 0)
    assert oracle.ulp_diff(a[5:], b[5:]) == (1, 1)
