"""Exact-rational helpers for pinning the oracle.  No oracle code is used here.

Everything is computed with Python's ``fractions.Fraction`` so that a result is the
mathematical one, then rounded to binary32 by an explicit nearest-even search.
"""
from fractions import Fraction

import numpy as np


def f32_to_fraction(v):
    return Fraction(float(np.float32(v)))


def round_to_f32(fr):
    """Correctly rounded (nearest, ties to even) binary32 of a Fraction."""
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    guess = np.float32(float(a))  # within one step of the answer
    cands = {guess, np.nextafter(guess, np.float32(np.inf), dtype=np.float32),
             np.nextafter(guess, np.float32(0.0), dtype=np.float32)}
    best, bd = None, None
    for c in cands:
        d = abs(Fraction(float(c)) - a)
        even = (int(np.float32(c).view(np.uint32)) & 1) == 0
        if best is None or d < bd or (d == bd and even):
            best, bd = c, d
    return np.float32(sign) * np.float32(best)


def tree_walk_value(kind, field):
    """Value of a 7-bit magnitude field by literally reading its bits (Sec. 3.1).

    kind 0 dynamic tree: leading zeros n -> 10^-n, flag bit, remaining bits bisect (0.1, 1).
    kind 1 linear: the field counts equal steps from 0 to 1.
    kind 2 static tree: 3 exponent bits (larger = bigger decade, top decade 10^0),
    4 bits bisect (0.1, 1).
    kind 3 mantissa: 3 exponent bits as in the static tree, 4 bits are the integer mantissa 0..15,
    which counts tenths of the decade: m * 10^(E-7) / 10.
    The value of a tree path is the middle of the interval the path ends in.
    """
    bits = [(field >> (6 - i)) & 1 for i in range(7)]
    if kind == 1:
        return Fraction(field, 127)
    if kind == 3:
        e = bits[0] * 4 + bits[1] * 2 + bits[2]
        m = bits[3] * 8 + bits[4] * 4 + bits[5] * 2 + bits[6]
        return Fraction(m, 10) * Fraction(1, 10 ** (7 - e))
    if kind == 0:
        n = 0
        while n < 7 and bits[n] == 0:
            n += 1
        if n == 7:
            return Fraction(0)
        path = bits[n + 1:]
        decade = Fraction(1, 10 ** n)
    else:
        e = bits[0] * 4 + bits[1] * 2 + bits[2]
        path = bits[3:]
        decade = Fraction(1, 10 ** (7 - e))
    lo, hi = Fraction(1, 10), Fraction(1)
    for b in path:
        mid = (lo + hi) / 2
        if b:
            lo = mid
        else:
            hi = mid
    return (lo + hi) / 2 * decade


def codebook_exact(kind):
    """256 Fractions: magnitudes by tree walk, upper half negated."""
    mags = [tree_walk_value(kind, j) for j in range(128)]
    return mags + [-m for m in mags]


def nearest_code_exact(cb_f32_fractions, cb_signbits, xn_fraction, xn_signbit):
    """Exact nearest code with the tie rules: lower magnitude, then matching sign bit."""
    best = None
    for c in range(256):
        d = abs(xn_fraction - cb_f32_fractions[c])
        m = abs(cb_f32_fractions[c])
        key = (d, m, 0 if cb_signbits[c] == xn_signbit else 1)
        if best is None or key < best[0]:
            best = (key, c)
    return best[1]
