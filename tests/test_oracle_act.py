"""Pins for the oracle's activation bounds (GELU-erf, SiLU, Mul/Add, ReLU; operators
of App. A.3, templates from the primitive rule of Sec. 3.1): dense sweeps of
binary32 inputs against binary64 / 60-digit references, special values."""
from fractions import Fraction

import mpmath as mp
import numpy as np
import pytest
from scipy import special

from exact import frac

mp.mp.dps = 60
U = 2.0 ** -24
f32 = np.float32


def _sweep(lo, hi, stride):
    b0 = np.array([lo], f32).view(np.uint32)[0]
    b1 = np.array([hi], f32).view(np.uint32)[0]
    pos = np.arange(b0, b1, stride, dtype=np.uint32).view(f32)
    return np.concatenate([pos, -pos, np.array([hi, -hi], f32)])


def _gelu_run(x, theta):
    kappa = f32(1.0 / np.sqrt(2.0))
    t = (x * kappa).astype(f32)
    g = (special.erf(t.astype(np.float64)) * (1 + theta)).astype(f32)     # erf within 2u
    h = (f32(1) + g).astype(f32)
    p = (f32(0.5) * x).astype(f32)
    return (p * h).astype(f32)


def test_constants_used_by_gelu():
    assert mp.mpf(float.fromhex("0x1.6a09e667f3bcdp-1")) > 1 / mp.sqrt(2) > mp.mpf(float.fromhex("0x1.6a09e667f3bccp-1"))
    up = float.fromhex("0x1.20dd750429b6ep+0")
    assert mp.mpf(up) > 2 / mp.sqrt(mp.pi) > mp.mpf(np.nextafter(up, 0.0))


@pytest.mark.parametrize("theta", [0.0, 0.99 * U, -0.99 * U])
def test_gelu_bound_is_sound_on_a_dense_sweep(oracle_mod, theta):
    x = _sweep(1e-30, 40.0, 2003)
    y = _gelu_run(x, theta)
    tau = oracle_mod.bound_act(oracle_mod.GELU_ERF, x, y).astype(np.float64)
    xd = x.astype(np.float64)
    ystar = 0.5 * xd * special.erfc(-xd / np.sqrt(2.0))
    err = np.abs(y.astype(np.float64) - ystar)
    slack = 1e-15 * np.abs(ystar)                      # accuracy of the binary64 reference
    assert np.all(err <= tau + slack)
    # tightness: the bound is a handful of u times the magnitudes involved
    assert np.all(tau <= 8 * U * np.maximum(np.abs(xd), np.abs(y)) + 1e-300)
    assert (err / np.maximum(tau, 1e-300)).max() > 0.15


def test_gelu_against_60_digits_and_special_values(oracle_mod):
    rng = np.random.Generator(np.random.Philox(21))
    x = (rng.standard_normal(400) * 3).astype(f32)
    y = _gelu_run(x, 0.0)
    tau = oracle_mod.bound_act(oracle_mod.GELU_ERF, x, y)
    for xi, yi, ti in zip(x, y, tau):
        xs = mp.mpf(float(xi))
        ystar = xs / 2 * (1 + mp.erf(xs / mp.sqrt(2)))
        assert abs(mp.mpf(float(yi)) - ystar) <= mp.mpf(float(ti))
    z = np.zeros(3, f32)
    assert np.all(oracle_mod.bound_act(oracle_mod.GELU_ERF, z, z) == 0)
    # the erf-sensitivity part is even in x: same y magnitude, opposite x
    xa = np.array([0.3, 1.0, 2.5], f32); ya = np.array([0.1, 0.2, 0.3], f32)
    assert np.array_equal(oracle_mod.bound_act(oracle_mod.GELU_ERF, xa, ya),
                          oracle_mod.bound_act(oracle_mod.GELU_ERF, -xa, -ya))
    # closed form at one point, evaluated with 60 digits
    x1 = f32(1.25); y1 = _gelu_run(np.array([x1]), 0.0)[0]
    u = mp.mpf(2) ** -24
    ts = mp.mpf(float(x1)) / mp.sqrt(2)
    E_t = (2 * u + u * u) * ts
    Gp = 2 / mp.sqrt(mp.pi) * mp.exp(-(ts - E_t) ** 2)
    A = min(mp.mpf(1), 2 / mp.sqrt(mp.pi) * ts * (1 + 4 * u))
    want = mp.mpf(float(x1)) / 2 * (Gp * E_t + 2 * u * A) + u * mp.mpf(float(y1)) * (1 + 1 / (1 - u))
    got = mp.mpf(float(oracle_mod.bound_act(oracle_mod.GELU_ERF, np.array([x1]), np.array([y1]))[0]))
    assert want <= got <= want * (1 + mp.mpf(2) ** -22)


@pytest.mark.parametrize("theta", [0.0, 0.99 * U, -0.99 * U])
def test_silu_bound_is_sound_on_a_dense_sweep(oracle_mod, theta):
    x = _sweep(1e-30, 87.0, 2003)
    xd = x.astype(np.float64)
    e = (np.exp(-xd) * (1 + theta)).astype(f32)        # exp within 2u
    D = (f32(1) + e).astype(f32)
    y = (x / D).astype(f32)
    tau = oracle_mod.bound_act(oracle_mod.SILU, x, y).astype(np.float64)
    ystar = xd / (1 + np.exp(-xd))
    err = np.abs(y.astype(np.float64) - ystar)
    assert np.all(err <= tau + 1e-15 * np.abs(ystar))
    u = Fraction(1, 2 ** 24)
    c1 = 2 * u / (1 - 2 * u)
    om = (c1 + u) / (1 - u)
    factor = om / (1 - u) + u
    k = np.argmax(np.abs(y))
    want = factor * abs(frac(y[k]))
    assert want <= frac(oracle_mod.bound_act(oracle_mod.SILU, x, y)[k]) <= want * (1 + Fraction(1, 2 ** 22))
    assert abs(float(factor) / U - 4.0) < 1e-5         # about (c_exp + 2) u |y|


def test_mul_add_relu(oracle_mod):
    rng = np.random.Generator(np.random.Philox(22))
    a = rng.standard_normal(3000).astype(f32)
    b = (rng.standard_normal(3000) * 7).astype(f32)
    for kind, y in ((oracle_mod.MUL, (a * b).astype(f32)), (oracle_mod.ADD, (a + b).astype(f32))):
        tau = oracle_mod.bound_act(kind, a, y, x2=b)
        for i in range(0, 3000, 7):
            exact = frac(a[i]) * frac(b[i]) if kind == oracle_mod.MUL else frac(a[i]) + frac(b[i])
            assert abs(frac(y[i]) - exact) <= frac(tau[i])
            want = Fraction(1, 2 ** 24) * abs(frac(y[i]))
            assert frac(tau[i]) >= want
            assert frac(tau[i]) <= want * (1 + Fraction(1, 2 ** 22)) or tau[i] <= np.float32(1e-44)
    y = np.maximum(a, 0)
    assert np.all(oracle_mod.bound_act(oracle_mod.RELU, a, y) == 0)


# ---- GELU, tanh form -----------------------------------------------------------------------------

def _gelu_tanh_run(x, theta, horner):
    """The binary32 algorithm with the tanh result pushed by the relative error theta."""
    beta = f32(np.sqrt(2.0 / np.pi)); a = f32(0.044715)
    if horner:
        inner = ((beta * x).astype(f32) * (f32(1) + (a * (x * x).astype(f32)).astype(f32)).astype(f32)).astype(f32)
    else:
        cube = ((x * x).astype(f32) * x).astype(f32)
        inner = (beta * (x + (a * cube).astype(f32)).astype(f32)).astype(f32)
    t = (np.tanh(inner.astype(np.float64)) * (1 + theta)).astype(f32)
    t = np.clip(t, f32(-1), f32(1))
    h = (f32(1) + t).astype(f32)
    return ((f32(0.5) * x).astype(f32) * h).astype(f32)


def _gelu_tanh_exact(xv):
    xs = mp.mpf(float(xv))
    return xs / 2 * (1 + mp.tanh(mp.sqrt(2 / mp.pi) * (xs + mp.mpf("0.044715") * xs ** 3)))


def test_constants_used_by_gelu_tanh():
    b = mp.sqrt(2 / mp.pi)
    assert mp.mpf(float.fromhex("0x1.9884533d43650p-1")) < b < mp.mpf(float.fromhex("0x1.9884533d43651p-1"))
    a = mp.mpf("0.044715")
    assert mp.mpf(float.fromhex("0x1.6e4e26d4801f7p-5")) < a < mp.mpf(float.fromhex("0x1.6e4e26d4801f8p-5"))


@pytest.mark.parametrize("theta,horner", [(0.0, False), (1.99 * U, False), (-1.99 * U, True), (0.0, True)])
def test_gelu_tanh_bound_is_sound_on_a_dense_sweep(oracle_mod, theta, horner):
    x = _sweep(1e-30, 30.0, 4001)
    y = _gelu_tanh_run(x, theta, horner)
    tau = oracle_mod.bound_act(oracle_mod.GELU_TANH, x, y)
    worst = mp.mpf(0)
    for xi, yi, ti in zip(x[::7], y[::7], tau[::7]):
        err = abs(mp.mpf(float(yi)) - _gelu_tanh_exact(xi))
        assert err <= mp.mpf(float(ti)), (xi, yi, ti)
        if ti > 0:
            worst = max(worst, err / mp.mpf(float(ti)))
    assert worst > 0.15
    # tightness: a handful of u times the magnitudes involved (7 roundings of p at sech^2 p <= 1,
    # p <= 1.2 |x| where it matters, the tanh accuracy, two fresh roundings)
    xd = np.abs(x.astype(np.float64))
    assert np.all(tau <= 12 * U * np.maximum(xd, np.abs(y)) + 1e-300)


def test_gelu_tanh_closed_form_special_values_and_limits(oracle_mod):
    o = oracle_mod
    z = np.zeros(3, f32)
    assert np.all(o.bound_act(o.GELU_TANH, z, z) == 0)
    xa = np.array([0.3, 1.0, 2.5], f32); ya = np.array([0.1, 0.2, 0.3], f32)
    assert np.array_equal(o.bound_act(o.GELU_TANH, xa, ya), o.bound_act(o.GELU_TANH, -xa, -ya))
    # the formula at a few points with 60 digits
    u = mp.mpf(2) ** -24
    g7 = 7 * u / (1 - 7 * u)
    for xv in (0.01, 0.75, 1.25, 3.0, 9.0):
        x1 = f32(xv); y1 = _gelu_tanh_run(np.array([x1]), 0.0, False)[0]
        xs = mp.mpf(float(x1))
        ps = mp.sqrt(2 / mp.pi) * (xs + mp.mpf("0.044715") * xs ** 3)
        E_p = g7 * ps
        Gp = 1 / mp.cosh(max(mp.mpf(0), ps - E_p)) ** 2
        A = min(mp.mpf(1), ps * (1 + g7))
        want = xs / 2 * (Gp * E_p + 4 * u * A) + u * mp.mpf(float(y1)) * (1 + 1 / (1 - u))
        got = mp.mpf(float(o.bound_act(o.GELU_TANH, np.array([x1]), np.array([y1]))[0]))
        assert want <= got <= want * (1 + mp.mpf(2) ** -22), xv
    # far out the sensitivity term is gone: (|x|/2) c_tanh u + 2u|y|, and a looser tanh moves it
    x = np.array([20.0], f32); y = x.copy()
    t = float(o.bound_act(o.GELU_TANH, x, y)[0])
    assert abs(t / (20.0 / 2 * 4 * U + 2 * U * 20.0) - 1) < 1e-6
    assert o.bound_act(o.GELU_TANH, x, y, model=o.Model(c_tanh=8.0))[0] > t
