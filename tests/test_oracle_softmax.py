"""Pins for the oracle's softmax bound: the printed template of Sec. 3.1 at first
order, brute-force soundness against a 60-digit evaluation, closed form on a
uniform row, masking, equivariance and monotonicity."""
import math
from fractions import Fraction

import mpmath as mp
import numpy as np
import pytest

from exact import all_fp32_sums, f32_round, frac, up32

mp.mp.dps = 60
U = 2.0 ** -24


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _to_frac(m):
    """mpmath value -> Fraction (exact for the stored binary significand)."""
    m = mp.mpf(m)
    man, exp = int(m.man), int(m.exp)
    v = Fraction(man) * (Fraction(2) ** exp)
    return -v if m._mpf_[0] else v


def _paper_template(x, gam):
    """Sec. 3.1 per-step bounds, evaluated in binary64 exactly as printed."""
    x = np.asarray(x, np.float64)
    m = x.max()
    z = x - m
    e = np.exp(z)
    S = e.sum()
    y = e / S
    eps_z = U * (np.abs(x) + abs(m))
    eps_e = e * eps_z + 2 * U * e
    eps_S = gam * e.sum() + (gam + 1) * eps_e.sum()
    return eps_e / S + e * eps_S / S ** 2 + U * y, y


@pytest.mark.parametrize("n", [2, 8, 128, 2048])
def test_reduces_to_printed_template_at_first_order(oracle_mod, n):
    rng = _rng(300 + n)
    x = (rng.standard_normal((6, n)) * 3).astype(np.float32)
    gam = oracle_mod.gamma(n - 1)
    for r in range(x.shape[0]):
        tp, y = _paper_template(x[r], gam)
        tau = oracle_mod.bound_softmax(x[r:r + 1], y.astype(np.float32)[None])[0]
        ratio = tau.astype(np.float64) / tp
        amax = 2 * U * np.abs(x[r]).max()
        assert ratio.min() >= 1 - 4 * U          # y is rounded to binary32 before use
        assert ratio.max() <= 1 + 4 * (n * U + amax) + 4 * U


def _canonical_runs(x, rng, c_exp=2.0):
    """Binary32 executions of m, z, e, S, y with exp within c_exp*u and every
    summation order; yields the output vectors."""
    m = np.max(x)
    z = [np.float32(v - m) for v in x]
    e = []
    for zz in z:
        theta = (c_exp - 1.0) * U * 0.99 * rng.uniform(-1, 1)
        e.append(f32_round(_to_frac(mp.exp(mp.mpf(float(zz))) * (1 + mp.mpf(theta)))))
    for S in sorted(all_fp32_sums(e)):
        yield np.array([np.float32(v / np.float32(S)) for v in e], np.float32)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_softmax_bound_is_sound(oracle_mod, n):
    rng = _rng(400 + n)
    for trial in range(12):
        x = (rng.standard_normal(n) * rng.choice([0.5, 4.0, 12.0])).astype(np.float32)
        if x.min() - x.max() < -80:      # exp would underflow: outside the model of App. A.1
            continue
        ex = [mp.exp(mp.mpf(float(v)) - mp.mpf(float(x.max()))) for v in x]
        ystar = [v / mp.fsum(ex) for v in ex]
        for y in _canonical_runs(x, rng):
            tau = oracle_mod.bound_softmax(x[None], y[None])[0]
            for i in range(n):
                err = abs(mp.mpf(float(y[i])) - ystar[i])
                assert err <= mp.mpf(float(tau[i])), (x, y, i)
            # first-order magnitude: not absurdly loose either
            assert np.all(tau <= (n + 8) * 4 * U * np.maximum(y, 1e-30) * (1 + np.abs(x).max()))


def test_uniform_row_closed_form(oracle_mod):
    for n, c in ((4, 0.0), (128, 1.5), (1000, -7.25)):
        x = np.full((1, n), c, np.float32)
        y32 = np.float32(1) / np.float32(n)
        tau = oracle_mod.bound_softmax(x, np.full((1, n), y32, np.float32))[0]
        u = Fraction(1, 2 ** 24)
        G = (n - 1) * u / (1 - (n - 1) * u)
        a = u * (2 * abs(Fraction(c)))
        rho = (a * (1 + a) + 2 * u) / (1 - 2 * u)
        q = frac(y32) / (1 - u)
        sigma = n * q * (G + (1 + G) * rho)
        want = q * rho + q * (1 + rho) * sigma / (1 - sigma) + u * frac(y32)
        w32 = up32(want)
        assert np.all((tau == w32) | (tau == np.nextafter(w32, np.float32(np.inf))))
        assert frac(tau[0]) >= want


def test_masking_nan_rows_and_equivariance(oracle_mod):
    rng = _rng(5)
    n = 12
    x = rng.standard_normal((3, n)).astype(np.float32)
    x[0, 7:] = -np.inf                       # causal-style mask
    x[1, :] = -np.inf                        # fully masked row
    e = np.exp(x - np.where(np.isfinite(x.max(1, keepdims=True)), x.max(1, keepdims=True), 0))
    with np.errstate(invalid="ignore"):
        y = (e / e.sum(1, keepdims=True)).astype(np.float32)
    y[1] = 0
    tau = oracle_mod.bound_softmax(x, y)
    assert np.all(tau[0, 7:] == 0) and np.all(tau[0, :7] > 0)
    assert np.all(np.isnan(tau[1]))
    assert np.all(np.isfinite(tau[2]))
    # a masked row of n columns equals... not the unmasked short row: k stays n-1
    short = oracle_mod.bound_softmax(x[0:1, :7], y[0:1, :7])[0]
    assert np.all(tau[0, :7] > short)
    # permutation equivariance
    p = rng.permutation(n)
    assert np.array_equal(oracle_mod.bound_softmax(x[2:3, p], y[2:3, p])[0], tau[2, p])
    # NaN or +inf input poisons the row
    xb = x[2:3].copy(); xb[0, 3] = np.nan
    assert np.all(np.isnan(oracle_mod.bound_softmax(xb, y[2:3])))


def test_monotone_in_constants_and_shift(oracle_mod):
    rng = _rng(6)
    n = 64
    x = rng.standard_normal((1, n)).astype(np.float32)
    e = np.exp(x.astype(np.float64) - x.max())
    y = (e / e.sum()).astype(np.float32)
    base = oracle_mod.bound_softmax(x, y)
    assert np.all(oracle_mod.bound_softmax(x, y, model=oracle_mod.Model(c_exp=4.0)) > base)
    assert np.all(oracle_mod.bound_softmax(x + np.float32(64), y) > base)   # |x|, |m| grow
    x2 = np.concatenate([x, np.full((1, n), -np.inf, np.float32)], axis=1)
    y2 = np.concatenate([y, np.zeros((1, n), np.float32)], axis=1)
    assert np.all(oracle_mod.bound_softmax(x2, y2)[0, :n] > base[0])        # larger n
    assert np.all(oracle_mod.bound_softmax(x, y, model=oracle_mod.Model(mode=1)) <= base)


def test_sigma_at_least_one_gives_nan(oracle_mod):
    # absurd intrinsic error makes the denominator bound collapse: no finite bound
    x = np.zeros((1, 4), np.float32)
    y = np.full((1, 4), 0.25, np.float32)
    tau = oracle_mod.bound_softmax(x, y, model=oracle_mod.Model(c_exp=2.0 ** 23))
    assert np.all(np.isnan(tau))
