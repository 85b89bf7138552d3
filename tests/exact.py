"""Exact-arithmetic helpers for pinning the oracle: binary32 values are dyadic
rationals, so |computed - exact| can be evaluated without any rounding."""
from fractions import Fraction
from itertools import combinations

import numpy as np

U = Fraction(1, 2 ** 24)


def frac(x):
    """Exact rational value of a binary32/binary64 number."""
    return Fraction(float(x))


def f32_round(q):
    """Round a rational to binary32, round-to-nearest ties-to-even (no overflow handling)."""
    q = Fraction(q)
    if q == 0:
        return np.float32(0.0)
    s = -1 if q < 0 else 1
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    ulp_exp = max(e, -126) - 23
    m = a / (Fraction(2) ** ulp_exp)
    fl = m.numerator // m.denominator
    rem = m - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (fl & 1)):
        fl += 1
    val = s * fl * Fraction(2) ** ulp_exp
    out = np.float32(float(val))
    assert Fraction(float(out)) == val
    return out


def all_fp32_sums(values):
    """Every binary32 result obtainable by summing `values` (np.float32) pairwise in any
    order / association: repeatedly replace two partial sums by their rounded sum."""
    seen = {}

    def rec(items):
        key = tuple(sorted(float(v) for v in items))
        if key in seen:
            return seen[key]
        if len(items) == 1:
            res = {float(items[0])}
        else:
            res = set()
            for i, j in combinations(range(len(items)), 2):
                rest = [items[k] for k in range(len(items)) if k != i and k != j]
                rest.append(np.float32(items[i] + items[j]))
                res |= rec(rest)
        seen[key] = res
        return res

    return rec([np.float32(v) for v in values])


def up32(q):
    """Smallest binary32 >= rational q (q >= 0)."""
    f = f32_round(q)
    if frac(f) < q:
        f = np.nextafter(f, np.float32(np.inf))
    return f
