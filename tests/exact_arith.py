"""Exact rational arithmetic with correct rounding to binary32, for brute-force pins of the oracle."""
from fractions import Fraction

import numpy as np


def exact_round_f32(q: Fraction) -> np.float32:
    """Correctly rounded binary32 of a rational, by exact neighbour comparison
    (no double rounding): start from the double-rounded guess and move to
    whichever neighbour is strictly closer; break ties to even."""
    g = np.float32(float(q))
    while True:
        lo = np.nextafter(g, np.float32(-np.inf))
        hi = np.nextafter(g, np.float32(np.inf))
        dg, dl, dh = (abs(Fraction(float(t)) - q) for t in (g, lo, hi))
        even_g = (int(np.array([g]).view(np.uint32)[0]) & 1) == 0
        if dl < dg or (dl == dg and not even_g):
            g = lo
        elif dh < dg or (dh == dg and not even_g):
            g = hi
        else:
            return g


def fr(x) -> Fraction:
    """The exact value of a binary32/binary64 number."""
    return Fraction(float(x))
