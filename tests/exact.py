"""Exact-rational helpers for pinning the oracle: they use Python's Fraction and
CPython's correctly rounded Fraction -> float conversion, nothing from oracle/."""
from fractions import Fraction

import numpy as np


def fma64(a, b, c):
    """Correctly rounded a*b+c in FP64 (exact rational sum, one rounding)."""
    return float(Fraction(a) * Fraction(b) + Fraction(c))


def nearest_in(candidates, exact, is_even):
    """Nearest candidate to the rational `exact`; a tie goes to the candidate is_even() accepts."""
    best = None
    for v in candidates:
        d = abs(Fraction(float(v)) - exact)
        if best is None or d < best[0] or (d == best[0] and is_even(v)):
            best = (d, v)
    return best[1]


def round32(exact):
    """Correctly rounded FP32 value of a rational: search the neighbours of a first guess."""
    exact = Fraction(exact)
    g = np.float32(float(exact))
    if not np.isfinite(g):
        return g
    cands = {g, np.nextafter(g, np.float32(np.inf)), np.nextafter(g, np.float32(-np.inf))}
    cands = [c for c in cands if np.isfinite(c)]

    def even(v):
        return (np.array(v, dtype=np.float32).view(np.uint32) & 1) == 0

    return nearest_in(cands, exact, even)


def fma32(a, b, c):
    return round32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


def e4m3_table():
    """All finite e4m3fn values by the format's definition: (code, Fraction value)."""
    out = []
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            continue
        v = Fraction(m, 8) * Fraction(2) ** -6 if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
        out.append((code, -v if s else v))
    return out
