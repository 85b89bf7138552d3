"""Pins for the oracle's two projections (Sec. 4.4): the clip onto the theoretical set and the
order-statistic projection onto the empirical set.  The latter is held against a hand-worked
example, closed forms, membership in the admissible set (rank by rank, and through numpy's own
percentile routine), idempotence, and a brute force over every assignment of caps to elements
that shows the sorted assignment is the nearest admissible point."""
from fractions import Fraction
from itertools import permutations

import numpy as np
import pytest

from exact import frac

f32 = np.float32
GRID = np.array([1] + [5 * g for g in range(1, 20)] + [99, 100], dtype=np.float64)


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _linear_thr(top):
    """Thresholds of the cap curve C(r) = top r / 100."""
    return (GRID / 100.0 * top).astype(f32)


def test_clip_is_the_elementwise_clamp(oracle_mod):
    o = oracle_mod
    d = np.array([3.0, -3.0, 0.5, -0.25, 0.0, -0.0, np.inf, -np.inf, np.nan], f32)
    t = np.array([1.0, 1.0, 1.0, 0.125, 1.0, 1.0, 2.0, 2.0, 1.0], f32)
    out = o.project_clip(d, t)
    want = np.array([1.0, -1.0, 0.5, -0.125, 0.0, -0.0, 2.0, -2.0, np.nan], f32)
    assert np.array_equal(out, want, equal_nan=True)
    assert np.signbit(out[5]) and not np.signbit(out[4])
    rng = _rng(1)
    d = rng.standard_normal(5000).astype(f32)
    t = np.abs(rng.standard_normal(5000)).astype(f32)
    assert np.array_equal(o.project_clip(d, t), np.clip(d, -t, t))
    # a scaled bound: alpha tau in binary64, then the largest binary32 value not above it
    out = o.project_clip(np.full(3, 10.0, f32), np.full(3, 1.0, f32) / f32(3), alpha=0.1)
    cap = Fraction(float(f32(1.0) / f32(3))) * Fraction(0.1)
    assert np.all(out == out[0]) and frac(out[0]) <= cap < frac(np.nextafter(out[0], f32(np.inf)))
    with pytest.raises(ValueError):
        o.project_clip(d, t[:-1])
    with pytest.raises(ValueError):
        o.project_clip(d, t, alpha=-1.0)


def test_hand_worked_example(oracle_mod):
    """n = 4, C(r) = 4 r / 100: ranks 12.5, 37.5, 62.5, 87.5 per cent give caps 0.5, 1.5, 2.5, 3.5.
    Magnitudes sorted: 0.25 (index 1), 2 (index 3), 3 (index 2), 8 (index 0)."""
    o = oracle_mod
    out = o.project_empirical(np.array([8.0, -0.25, 3.0, -2.0], f32), _linear_thr(4.0))
    assert np.allclose(out, [3.5, -0.25, 2.5, -1.5], rtol=1e-6, atol=0)
    assert out[1] == f32(-0.25)                      # below its cap: bit-identical
    # n = 1: the single element sits at rank 50 per cent
    out = o.project_empirical(np.array([-9.0], f32), _linear_thr(4.0))
    assert np.isclose(out[0], -2.0, rtol=1e-6)


def test_cap_curve_against_numpy_interp_and_the_knots(oracle_mod):
    o = oracle_mod
    rng = _rng(2)
    thr = np.sort(np.abs(rng.standard_normal(22))).astype(f32)
    n = 1000
    k = np.arange(1, n + 1)
    got = o.cap_curve(k, n, thr, alpha=2.0)
    r = (k - 0.5) / n * 100.0
    want = np.interp(r, np.concatenate([[0.0], GRID]), np.concatenate([[0.0], thr.astype(np.float64) * 2.0]))
    assert np.allclose(got, want, rtol=1e-12, atol=0)
    # ranks that land on knots (n = 200: r_k = (k - 1/2)/2 hits p = 5, 10, ... at k = 10.5?  no:
    # use n = 50, r_k = 2k - 1, which meets 1, 5, 15, 25, ... 95, 99)
    n = 50
    k = np.arange(1, n + 1)
    got = o.cap_curve(k, n, thr)
    for j, p in enumerate(GRID):
        hit = np.nonzero(2 * k - 1 == p)[0]
        for h in hit:
            assert np.isclose(got[h], float(thr[j]), rtol=1e-15)
    # through the origin: the first segment is a line from (0, 0) to (1, thr_1)
    n = 10000
    assert np.isclose(o.cap_curve([1], n, thr)[0], float(thr[0]) * 0.005, rtol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_result_is_admissible_nearest_and_idempotent(oracle_mod, seed):
    o = oracle_mod
    rng = _rng(10 + seed)
    n = int(rng.integers(50, 4000))
    d = (rng.standard_normal(n) * 1e-5).astype(f32)
    alpha = float(rng.choice([1.0, 2.0, 3.0]))
    thr = np.sort(np.abs(rng.standard_normal(22)) * (0.7e-5 / alpha)).astype(f32)
    out = o.project_empirical(d, thr, alpha)
    # sign and shape restored, magnitudes never grow, untouched elements bit-identical
    assert out.shape == d.shape and np.array_equal(np.signbit(out), np.signbit(d))
    assert np.all(np.abs(out) <= np.abs(d))
    caps = np.maximum.accumulate(o.cap_curve(np.arange(1, n + 1), n, thr, alpha))
    srt = np.sort(np.abs(out))
    assert np.all(srt.astype(np.float64) <= caps)                     # admissible, rank by rank
    # and every clipped order statistic sits at its cap (to binary32 rounding): nothing is
    # clipped further than needed
    a_sorted = np.sort(np.abs(d))
    was = a_sorted.astype(np.float64) > caps
    assert was.any() and not was.all()
    # (clipping keeps the order: min(a_(k), c_k) is nondecreasing in k)
    assert np.allclose(srt[was], caps[was], rtol=2e-7, atol=1e-45)
    assert np.array_equal(srt[~was], a_sorted[~was])
    # numpy's percentile of the result stays under the curve at the ranks' own positions
    q = np.percentile(np.abs(out).astype(np.float64), (np.arange(1, n + 1) - 0.5) / n * 100.0,
                      method="hazen")
    assert np.all(q <= caps * (1 + 1e-12))
    # idempotent
    assert np.array_equal(o.project_empirical(out, thr, alpha), out)


def test_sorted_assignment_is_the_nearest_admissible_point(oracle_mod):
    """Delta is admissible iff some assignment of the caps c_1 <= ... <= c_n to the elements
    dominates its magnitudes; for a fixed assignment the nearest point clips element i to its cap.
    Brute force over all n! assignments: none is closer than the oracle's result."""
    o = oracle_mod
    rng = _rng(3)
    for trial in range(40):
        n = int(rng.integers(2, 7))
        d = rng.standard_normal(n).astype(f32)
        thr = np.sort(np.abs(rng.standard_normal(22))).astype(f32) * f32(rng.uniform(0.2, 2.0))
        out = o.project_empirical(d, thr)
        caps = np.maximum.accumulate(o.cap_curve(np.arange(1, n + 1), n, thr))
        a = np.abs(d).astype(np.float64)
        best = min(sum((a[i] - min(a[i], caps[pi[i]])) ** 2 for i in range(n))
                   for pi in permutations(range(n)))
        dist = float(np.sum((d.astype(np.float64) - out.astype(np.float64)) ** 2))
        assert dist <= best * (1 + 1e-6) + 1e-30
        assert dist >= best * (1 - 1e-6) - 1e-30      # rounding down to binary32 only


def test_closed_forms_and_degenerate_inputs(oracle_mod):
    o = oracle_mod
    rng = _rng(4)
    d = rng.standard_normal(777).astype(f32)
    # huge caps: identity; zero caps: everything to (signed) zero
    assert np.array_equal(o.project_empirical(d, np.full(22, 1e30, f32)), d)
    z = o.project_empirical(d, np.zeros(22, f32))
    assert np.all(z == 0) and np.array_equal(np.signbit(z), np.signbit(d))
    # all magnitudes equal: ranks follow the index order (stable), so the output is the cap
    # sequence itself wherever it is below the common magnitude
    n = 64
    e = np.full(n, 5.0, f32); e[::2] *= -1
    thr = _linear_thr(8.0)
    out = o.project_empirical(e, thr)
    caps = o.cap_curve(np.arange(1, n + 1), n, thr)
    assert np.allclose(np.abs(out), np.minimum(caps, 5.0), rtol=2e-7)
    assert np.all(np.diff(np.abs(out)) >= 0)
    # a threshold table that is not monotone: the running maximum keeps the caps nondecreasing
    thr = _linear_thr(8.0); thr[10:14] = 0.0
    out = o.project_empirical(np.full(2000, 100.0, f32), thr)
    assert np.all(np.diff(out) >= 0) and out[-1] > 7.9
    flat = out[(np.arange(2000) + 0.5) / 20.0 > 55.0][:100]
    # the running maximum is over the sampled ranks: the last one before the drop is 44.975 per
    # cent, so the plateau is 8 x 0.44975, not the knot's 3.6 that no rank samples
    assert np.allclose(flat, 8.0 * 0.44975, rtol=1e-6) and np.all(flat < f32(3.6))
    # empty, NaN, infinity, signed zero
    assert o.project_empirical(np.zeros((0, 3), f32), thr).shape == (0, 3)
    s = np.array([np.nan, -np.inf, 0.0, -0.0, 1e-3, np.inf], f32)
    out = o.project_empirical(s, _linear_thr(6.0))
    assert np.isnan(out[0]) and out[2] == 0 and np.signbit(out[3]) and not np.signbit(out[2])
    # ranks: 0.0 (1), -0.0 (2), 1e-3 (3), -inf (4), inf (5), nan (6); caps 6 (k - 1/2)/6 per cent
    assert out[4] == f32(1e-3) and np.isclose(out[1], -3.5, rtol=1e-6) and np.isclose(out[5], 4.5, rtol=1e-6)
    # shape is restored
    m = rng.standard_normal((4, 5, 6)).astype(f32)
    assert o.project_empirical(m, _linear_thr(1.0)).shape == (4, 5, 6)
    with pytest.raises(ValueError):
        o.project_empirical(d, np.ones(21, f32))
    with pytest.raises(ValueError):
        o.project_empirical(d, -np.ones(22, f32))
    with pytest.raises(ValueError):
        o.project_empirical(d, np.ones(22, f32), alpha=float("nan"))


def test_rounding_of_a_clipped_element_never_leaves_the_set(oracle_mod):
    o = oracle_mod
    thr = (np.sort(np.abs(_rng(5).standard_normal(22))) / 3.0).astype(f32)
    n = 300
    out = o.project_empirical(np.full(n, 1e6, f32), thr, alpha=1.0 / 3.0)
    caps = np.maximum.accumulate(o.cap_curve(np.arange(1, n + 1), n, thr, 1.0 / 3.0))
    for v, c in zip(out, caps):
        assert frac(v) <= frac(c) < frac(np.nextafter(v, f32(np.inf)))
