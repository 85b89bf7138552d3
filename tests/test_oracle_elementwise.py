"""Pins for the oracle's one-step element-wise kinds (Sub, Div, Sqrt, Rsqrt, Exp, Log, Sin, Cos,
Tanh, Pow, Sigmoid, exact operators; App. A.3) and for the rotary-embedding bound: the factor as
an exact rational, soundness against 50-digit references for library outputs pushed to the edge
of their accuracy contract, real binary32 evaluations, and for the rotation the matmul bound of
the equivalent two-term dot products plus exact-rational brute force over evaluation orders."""
from fractions import Fraction

import mpmath as mp
import numpy as np
import pytest

from exact import all_fp32_sums, f32_round, frac, up32

mp.mp.dps = 50
U = Fraction(1, 2 ** 24)
f32 = np.float32


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _lib_kinds(o):
    m = o.Model()
    return {o.DIV: m.c_div, o.RSQRT: m.c_rsqrt, o.EXP: m.c_exp, o.LOG: m.c_log, o.SIN: m.c_sin,
            o.COS: m.c_cos, o.TANH: m.c_tanh, o.POW: m.c_pow}


def test_factor_of_every_kind_as_an_exact_rational(oracle_mod):
    o = oracle_mod
    y = np.array([1.0, -3.5, 1e-20, 65504.0, 2.0 ** -130, 0.0], f32)
    for kind in (o.SUB, o.SQRT, o.MUL, o.ADD):
        t = o.bound_act(kind, None, y)
        for yi, ti in zip(y, t):
            assert ti == up32(U * abs(frac(yi)))
    for kind, c in _lib_kinds(o).items():
        c = Fraction(c)
        f = c * U / (1 - c * U)
        t = o.bound_act(kind, None, y)
        for yi, ti in zip(y, t):
            want = up32(f * abs(frac(yi)))
            assert ti in (want, np.nextafter(want, f32(np.inf))) and frac(ti) >= f * abs(frac(yi))
    for kind in (o.EXACT, o.RELU):
        assert np.all(o.bound_act(kind, None, y) == 0)
    # the sigmoid shares the SiLU factor; a changed accuracy constant moves only its own kind
    assert np.array_equal(o.bound_act(o.SIGMOID, None, y), o.bound_act(o.SILU, None, y))
    loose = o.Model(c_log=6.0)
    assert np.all(o.bound_act(o.LOG, None, y[:4], model=loose) > o.bound_act(o.LOG, None, y[:4]))
    assert np.array_equal(o.bound_act(o.SIN, None, y, model=loose), o.bound_act(o.SIN, None, y))
    with pytest.raises(ValueError):
        o.bound_act(18, None, y)
    with pytest.raises(ValueError):
        o.bound_act(o.GELU_TANH, None, y)          # needs x


FUNCS = {
    "EXP": (lambda v: mp.exp(v), -80.0, 80.0),
    "LOG": (lambda v: mp.log(v), 1e-30, 1e30),
    "SIN": (lambda v: mp.sin(v), -100.0, 100.0),
    "COS": (lambda v: mp.cos(v), -100.0, 100.0),
    "TANH": (lambda v: mp.tanh(v), -12.0, 12.0),
    "RSQRT": (lambda v: 1 / mp.sqrt(v), 1e-30, 1e30),
}


@pytest.mark.parametrize("name", sorted(FUNCS))
def test_library_kinds_are_sound_at_the_edge_of_the_accuracy_contract(oracle_mod, name):
    """y = round-to-binary32 of y*(1 + s c u) stays inside the contract |y - y*| <= c u |y*| when it
    is rounded toward y*; for both signs s the bound computed from y alone must cover the error.
    s = -1 is the case that needs the 1/(1 - c u) closure."""
    o = oracle_mod
    kind = getattr(o, name)
    c = _lib_kinds(o)[kind]
    fn, lo, hi = FUNCS[name]
    rng = _rng(len(name))
    if lo > 0:
        xs = np.exp(rng.uniform(np.log(lo), np.log(hi), 300)).astype(f32)
    else:
        xs = rng.uniform(lo, hi, 300).astype(f32)
    cu = mp.mpf(c) * mp.mpf(2) ** -24
    worst = mp.mpf(0)
    for s in (+1, -1):
        ys = []
        stars = []
        for xv in xs:
            star = fn(mp.mpf(float(xv)))
            edge = star * (1 + s * cu)
            # nearest binary32 values around the edge; keep the one on the y* side of it
            cand = f32(float(edge))
            if abs(mp.mpf(float(cand)) - star) > cu * abs(star):
                cand = np.nextafter(cand, f32(float(star)))
            assert abs(mp.mpf(float(cand)) - star) <= cu * abs(star)
            ys.append(cand); stars.append(star)
        ys = np.array(ys, f32)
        tau = o.bound_act(kind, xs, ys)
        for yv, star, tv in zip(ys, stars, tau):
            err = abs(mp.mpf(float(yv)) - star)
            assert err <= mp.mpf(float(tv))
            if tv > 0:
                worst = max(worst, err / mp.mpf(float(tv)))
    assert worst > 0.9          # the contract's edge is nearly reached: the factor is not padded


def test_correctly_rounded_kinds_on_real_binary32_arithmetic(oracle_mod):
    o = oracle_mod
    rng = _rng(5)
    a = (rng.standard_normal(2000) * 10.0 ** rng.integers(-10, 10, 2000)).astype(f32)
    b = (rng.standard_normal(2000) * 10.0 ** rng.integers(-10, 10, 2000)).astype(f32)
    cases = [(o.SUB, a - b, [frac(p) - frac(q) for p, q in zip(a, b)]),
             (o.ADD, a + b, [frac(p) + frac(q) for p, q in zip(a, b)]),
             (o.MUL, a * b, [frac(p) * frac(q) for p, q in zip(a, b)])]
    for kind, y, exact in cases:
        y = y.astype(f32)
        tau = o.bound_act(kind, a, y, x2=b)
        normal = np.abs(y) >= 2.0 ** -126
        for yi, ei, ti, ok in zip(y, exact, tau, normal):
            if ok:
                assert abs(frac(yi) - ei) <= frac(ti)
    pos = np.abs(a) + f32(1e-30)
    y = np.sqrt(pos).astype(f32)
    tau = o.bound_act(o.SQRT, pos, y)
    for p, yi, ti in zip(pos[:300], y, tau):
        assert abs(mp.mpf(float(yi)) - mp.sqrt(mp.mpf(float(p)))) <= mp.mpf(float(ti))
    # division as numpy performs it is correctly rounded: inside the bound for any c_div >= 1
    q = (a / b).astype(f32)
    tau = o.bound_act(o.DIV, a, q, x2=b)
    for p, r, yi, ti in zip(a[:300], b[:300], q, tau):
        if abs(yi) >= 2.0 ** -126 and np.isfinite(yi):
            assert abs(frac(yi) - frac(p) / frac(r)) <= frac(ti)


# ---- rotary embedding -------------------------------------------------------------------------

def _rope_ref_pairs(d, interleaved):
    h = d // 2
    return [(2 * j, 2 * j + 1) if interleaved else (j, j + h) for j in range(h)]


@pytest.mark.parametrize("interleaved", [False, True])
def test_rope_is_the_matmul_bound_of_two_term_dot_products(oracle_mod, interleaved):
    o = oracle_mod
    rng = _rng(31)
    rows, d, npos, inner = 12, 8, 3, 2
    x = rng.standard_normal((rows, d)).astype(f32)
    ang = rng.uniform(-3, 3, (npos, d // 2))
    cs, sn = np.cos(ang).astype(f32), np.sin(ang).astype(f32)
    tau = o.bound_rope(x, cs, sn, inner=inner, interleaved=interleaved)
    for r in range(rows):
        t = (r // inner) % npos
        for j, (a, b) in enumerate(_rope_ref_pairs(d, interleaved)):
            A = np.array([[x[r, a], x[r, b]]], f32)
            Wa = np.array([[cs[t, j], -sn[t, j]]], f32)      # y_a = x_a cos - x_b sin
            Wb = np.array([[sn[t, j], cs[t, j]]], f32)       # y_b = x_a sin + x_b cos
            assert tau[r, a] == o.bound_linear(A, Wa)[0, 0]
            assert tau[r, b] == o.bound_linear(A, Wb)[0, 0]


def test_rope_closed_form_and_table_indexing(oracle_mod):
    o = oracle_mod
    g2 = 2 * U / (1 - 2 * U)
    x = np.ones((4, 4), f32)
    cs = np.array([[1, 1], [0, 0]], f32); sn = np.array([[1, 1], [2, 2]], f32)
    t = o.bound_rope(x, cs, sn, inner=2)          # rows 0,1 -> table 0; rows 2,3 -> table 1
    assert np.all(t[:2] == up32(g2 * 2)) and np.all(t[2:] == up32(g2 * 2))
    t = o.bound_rope(x * f32(3), cs, sn, inner=1)  # rows alternate tables 0,1,0,1
    assert np.all(t[0::2] == up32(g2 * 6)) and np.all(t[1::2] == up32(g2 * 6))
    # a zero angle leaves x unrotated: the bound is Gamma(2)|x| (one exact product, k stays 2)
    cs = np.ones((1, 2), f32); sn = np.zeros((1, 2), f32)
    xr = np.array([[1.5, -2.0, 0.25, 8.0]], f32)
    assert np.array_equal(o.bound_rope(xr, cs, sn), np.array([[up32(g2 * abs(frac(v))) for v in xr[0]]], f32))
    with pytest.raises(ValueError):
        o.bound_rope(np.ones((1, 3), f32), np.ones((1, 1), f32), np.ones((1, 1), f32))


def test_rope_bound_is_sound_for_every_evaluation(oracle_mod):
    """Separately rounded products summed either way, and both fused forms."""
    o = oracle_mod
    rng = _rng(33)
    worst = 0.0
    for trial in range(200):
        xa, xb = (rng.standard_normal(2) * 2.0 ** rng.integers(-5, 6)).astype(f32)
        th = rng.uniform(-3.2, 3.2)
        c, s = f32(np.cos(th)), f32(np.sin(th))
        x = np.array([[xa, xb]], f32)
        tau = o.bound_rope(x, np.array([[c]], f32), np.array([[s]], f32))[0]
        for (p1, q1, p2, q2, sign), tv in (((xa, c, xb, s, -1), tau[0]), ((xb, c, xa, s, +1), tau[1])):
            exact = frac(p1) * frac(q1) + sign * frac(p2) * frac(q2)
            t1, t2 = frac(p1) * frac(q1), sign * frac(p2) * frac(q2)
            results = [f32_round(frac(f32_round(t1)) + frac(f32_round(t2))),     # two products, one add
                       f32_round(t1 + frac(f32_round(t2))),                       # fma(p1, q1, fl(p2 q2))
                       f32_round(frac(f32_round(t1)) + t2)]                       # fma(p2, q2, fl(p1 q1))
            for r in results:
                err = abs(frac(r) - exact)
                assert err <= frac(tv)
                if tv > 0:
                    worst = max(worst, float(err / frac(tv)))
    assert 0.2 < worst <= 1.0
