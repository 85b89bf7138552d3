"""Pins for the oracle's gamma constants: closed forms of App. A.1 Eq. (gamma-def)
and the probabilistic constant and confidence printed in Sec. 3.1."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

HERE = os.path.dirname(__file__)


def _rows():
    for line in open(os.path.join(HERE, "golden", "gamma_closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, a, b = map(int, line.split())
        yield k, Fraction(a, b)


def test_golden_file_matches_closed_form():
    u = Fraction(1, 2 ** 24)
    for k, g in _rows():
        assert g == k * u / (1 - k * u)


def test_gamma_is_tight_upper_enclosure(oracle_mod):
    for k, g in _rows():
        v = oracle_mod.gamma(k)
        assert Fraction(v) >= g
        assert Fraction(float(np.nextafter(v, 0.0))) < g      # no more than one ulp above


def test_gamma_small_k_and_expansion(oracle_mod):
    u = 2.0 ** -24
    assert oracle_mod.gamma(0) == 0.0
    assert oracle_mod.gamma(-3) == 0.0
    for k in (1, 2, 3, 5, 100):
        g = oracle_mod.gamma(k)
        exact = Fraction(k, 2 ** 24) / (1 - Fraction(k, 2 ** 24))
        assert Fraction(g) >= exact
        # gamma_k = k u + O(u^2)  (App. A.1)
        assert 0 < g - k * u < 2 * (k * u) ** 2


def test_gamma_monotone_and_validity(oracle_mod):
    prev = 0.0
    for k in (1, 2, 10, 255, 256, 257, 4096, 10 ** 6, 2 ** 24 - 1):
        g = oracle_mod.gamma(k)
        assert g > prev
        prev = g
    assert math.isnan(oracle_mod.gamma(2 ** 24))          # k u = 1: constant undefined
    assert math.isnan(oracle_mod.gamma(2 ** 24 + 5))


def test_probabilistic_constant(oracle_mod):
    # Sec. 3.1: lambda = 4 gives about 4 u sqrt(k) at >= 99.93 % confidence.
    u = 2.0 ** -24
    md = oracle_mod.Model(mode=1, lam=4.0)
    for k in (16, 256, 4096, 8192):
        g = oracle_mod.gamma(k, md)
        first = 4 * u * math.sqrt(k)
        assert first < g < first * (1 + 1e-4)
        exact = math.expm1(4 * math.sqrt(k) * u + k * u * u / (1 - u))
        assert exact <= g <= exact * (1 + 1e-12)
    assert abs(oracle_mod.gamma(256, md) - 3.8147e-6) < 1e-9
    conf = 1 - 2 * math.exp(-(4.0 ** 2) * (1 - u) ** 2 / 2)
    assert 0.9993 <= conf < 0.9994
    # the probabilistic constant is far below the deterministic one at large k
    assert oracle_mod.gamma(8192, md) < oracle_mod.gamma(8192) / 20
