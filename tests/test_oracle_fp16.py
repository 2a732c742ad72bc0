"""Pins for the oracle's binary16 conversion (Section 3.2: half-precision
transfer).  None of these retype the oracle's routine: they check it against
the IEEE-754 definition of round-to-nearest-even evaluated in exact rational
arithmetic, against range boundaries derived by hand, and against numpy's own
conversion."""
from fractions import Fraction

import numpy as np
import pytest


def half_value(h: int) -> Fraction:
    """Exact value of a finite binary16 bit pattern, from the format definition."""
    s = -1 if h & 0x8000 else 1
    e = (h >> 10) & 0x1F
    m = h & 0x3FF
    assert e != 0x1F
    if e == 0:
        return s * Fraction(m, 1 << 24)
    return s * Fraction(1024 + m, 1024) * Fraction(2) ** (e - 15)


def f32_bits(x: float) -> int:
    return int(np.array([x], np.float32).view(np.uint32)[0])


def f32_from_bits(u: int) -> np.float32:
    return np.array([u], np.uint32).view(np.float32)[0]


def nearest_half_bruteforce(x: Fraction, table) -> int:
    """IEEE round-to-nearest-even over the positive finite halves plus the
    overflow rule: values at or beyond max + ulp/2 go to infinity."""
    sign = 0x8000 if x < 0 else 0
    ax = abs(x)
    top = Fraction(65504) + Fraction(16)          # 65520: halfway to 2^16
    if ax >= top:
        return sign | 0x7C00
    best, bestd = None, None
    for h, v in table:
        d = abs(v - ax)
        if bestd is None or d < bestd or (d == bestd and (h & 1) == 0):
            best, bestd = h, d
    return sign | best


def test_widen_is_exact_for_all_halves(oracle_mod):
    """All 2^16 halves: the oracle's widening equals the value the format
    defines (checked exactly) and equals numpy's widening bit for bit."""
    hs = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    wide = oracle_mod.unpack_fp16(hs.view(np.float16))
    ref = hs.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(wide), nan)
    assert np.array_equal(wide.view(np.uint32)[~nan], ref.view(np.uint32)[~nan])
    for h in list(range(0, 0x7C00, 37)) + [1, 0x3FF, 0x400, 0x7BFF, 0x8001, 0xFBFF]:
        assert Fraction(float(wide[h])) == half_value(h), hex(h)


def test_exhaustive_round_trip(oracle_mod):
    """widen then pack returns the same 16 bits for every non-NaN half; NaN
    stays NaN with its sign."""
    hs = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    wide = hs.view(np.float16).astype(np.float32)     # numpy's widening, not the oracle's
    back = oracle_mod.pack_fp16(wide).view(np.uint16)
    e = (hs >> 10) & 0x1F
    nan = (e == 0x1F) & ((hs & 0x3FF) != 0)
    assert np.array_equal(back[~nan], hs[~nan])
    bn = back[nan]
    assert np.all(((bn >> 10) & 0x1F) == 0x1F) and np.all((bn & 0x3FF) != 0)
    assert np.array_equal(bn & 0x8000, hs[nan] & 0x8000)


def test_every_tie_between_adjacent_halves(oracle_mod):
    """For each adjacent pair of non-negative finite halves (h, h+1) the
    binary32 midpoint is exactly representable.  It must go to the one with the
    even mantissa; one binary32 step below goes to h, one above to h+1.  The
    last pair's upper neighbour is 2^16, i.e. infinity after rounding."""
    lo = np.arange(0, 0x7C00, dtype=np.uint32)            # 0 .. 0x7BFF
    vlo = lo.astype(np.uint16).view(np.float16).astype(np.float64)
    vhi = np.empty_like(vlo)
    vhi[:-1] = vlo[1:]
    vhi[-1] = 65536.0
    mid64 = (vlo + vhi) / 2
    mid = mid64.astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), mid64)  # exactly representable
    below = np.nextafter(mid, np.float32(-np.inf))
    above = np.nextafter(mid, np.float32(np.inf))
    for sgn in (1.0, -1.0):
        sbit = 0 if sgn > 0 else 0x8000
        got_mid = oracle_mod.pack_fp16((sgn * mid).astype(np.float32)).view(np.uint16)
        got_lo = oracle_mod.pack_fp16((sgn * below).astype(np.float32)).view(np.uint16)
        got_hi = oracle_mod.pack_fp16((sgn * above).astype(np.float32)).view(np.uint16)
        want_mid = np.where(lo % 2 == 0, lo, lo + 1).astype(np.uint16) | sbit
        assert np.array_equal(got_mid, want_mid)
        assert np.array_equal(got_lo, lo.astype(np.uint16) | sbit)
        assert np.array_equal(got_hi, (lo + 1).astype(np.uint16) | sbit)
    # 0x7BFF + 1 == 0x7C00 is infinity: covered by the last pair above.


BOUNDARY_CASES = [
    # (binary32 value, expected binary16 bits), each derived from the format:
    (65504.0, 0x7BFF),                       # largest finite half
    (65519.996, 0x7BFF),                     # just under the halfway point 65520
    (65520.0, 0x7C00),                       # halfway to 2^16, odd neighbour -> up -> inf
    (65536.0, 0x7C00),
    (3.0e38, 0x7C00),
    (-65520.0, 0xFC00),
    (2.0 ** -14, 0x0400),                    # smallest normal
    (2.0 ** -14 - 2.0 ** -25, 0x0400),       # tie between 0x3FF and 0x400 -> even (0x400)
    (2.0 ** -24, 0x0001),                    # smallest subnormal
    (2.0 ** -25, 0x0000),                    # tie between 0 and 0x0001 -> even (0)
    (-(2.0 ** -25), 0x8000),
    (1.5 * 2.0 ** -24, 0x0002),              # tie between 1 and 2 -> even (2)
    (2.5 * 2.0 ** -24, 0x0002),              # tie between 2 and 3 -> even (2)
    (2.0 ** -26, 0x0000),
    (0.0, 0x0000),
    (-0.0, 0x8000),
    (1.0, 0x3C00),
    (1.0 + 2.0 ** -11, 0x3C00),              # tie, even stays
    (1.0 + 3 * 2.0 ** -11, 0x3C02),          # tie, odd goes up
    (2047.5, 0x67FF + 1),                    # 2047 and 2048 are neighbours at ulp 1: tie -> 2048 (0x6800)
    (float("inf"), 0x7C00),
    (float("-inf"), 0xFC00),
]


@pytest.mark.parametrize("x,want", BOUNDARY_CASES)
def test_boundaries(oracle_mod, x, want):
    assert oracle_mod.f32_to_f16_bits(f32_bits(x)) == want


def test_nextafter_of_quarter_ulp_boundary(oracle_mod):
    up = np.nextafter(np.float32(2.0 ** -25), np.float32(1))
    assert oracle_mod.f32_to_f16_bits(f32_bits(up)) == 0x0001
    dn = np.nextafter(np.float32(65520.0), np.float32(0))
    assert oracle_mod.f32_to_f16_bits(f32_bits(dn)) == 0x7BFF


def test_float32_subnormals_flush_to_signed_zero(oracle_mod):
    for u in (0x00000001, 0x007FFFFF, 0x00400000):
        assert oracle_mod.f32_to_f16_bits(u) == 0x0000
        assert oracle_mod.f32_to_f16_bits(u | 0x80000000) == 0x8000


def test_nan_stays_nan_with_sign(oracle_mod):
    for u in (0x7FC00000, 0x7F800001, 0xFFC12345, 0x7FFFFFFF, 0xFF800001):
        h = oracle_mod.f32_to_f16_bits(u)
        assert (h & 0x7C00) == 0x7C00 and (h & 0x03FF) != 0
        assert (h & 0x0200) != 0                      # quiet
        assert (h >> 15) == (u >> 31)


def test_against_exact_nearest_search(oracle_mod):
    """Independent definition: pick the nearest finite half by exact rational
    distance, ties to the even pattern, for random values across the range."""
    table = [(h, half_value(h)) for h in range(0, 0x7C00)]
    rng = np.random.default_rng(7)
    # a coarse table search per value is slow; restrict candidates by numpy's
    # ordering of halves (monotone in bit pattern for non-negative values)
    vals = np.concatenate([
        (rng.standard_normal(300) * 0.01).astype(np.float32),
        np.exp2(rng.uniform(-27, 17, 300)).astype(np.float32) * rng.choice([-1, 1], 300).astype(np.float32),
    ])
    allv = np.array([float(v) for _, v in table])
    for x in vals:
        fx = Fraction(float(x))
        i = int(np.searchsorted(allv, abs(float(x))))
        cand = table[max(0, i - 2): i + 2]
        want = nearest_half_bruteforce(fx, cand)
        if x < 0 or (x == 0 and np.signbit(x)):
            want |= 0x8000
        assert oracle_mod.f32_to_f16_bits(f32_bits(float(x))) == want, float(x)


def test_against_numpy_conversion_on_random_bit_patterns(oracle_mod):
    """Library special case: numpy's float32 -> float16 cast is IEEE RNE."""
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 1 << 32, 10_000_000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    got = oracle_mod.pack_fp16(x).view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    gn = got[nan]
    assert np.all((gn & 0x7C00) == 0x7C00) and np.all((gn & 0x3FF) != 0)


def test_gradient_like_values_hit_the_subnormal_range(oracle_mod):
    """With sigma = 0.01 about half a percent of gradients are below 2^-14 in
    magnitude, so gradual underflow matters for the benchmark inputs."""
    rng = np.random.default_rng(3)
    g = (rng.standard_normal(2_000_000) * 0.01).astype(np.float32)
    h = oracle_mod.pack_fp16(g)
    with np.errstate(over="ignore"):
        assert np.array_equal(h.view(np.uint16), g.astype(np.float16).view(np.uint16))
    sub = np.abs(g) < 2.0 ** -14
    assert 0.003 < sub.mean() < 0.007
    # relative error bound of RNE in the normal range: 2^-11
    w = h.astype(np.float32)
    assert np.all(np.abs(w[~sub] - g[~sub]) <= np.abs(g[~sub]) * 2.0 ** -11)
    assert np.all(np.abs(w[sub] - g[sub]) <= 2.0 ** -25)
