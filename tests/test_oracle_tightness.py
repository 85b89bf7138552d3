"""Tightness pins for the templates the paper does not print (LayerNorm, RMSNorm, GELU, SiLU:
operators of App. A.3, bounds derived from the primitive rule of Sec. 3.1).

The soundness pins (brute force over executions) exclude an under-estimate; the closed-form pins
re-evaluate the oracle's own chain, so a uniformly over-estimated term would pass them.  Here the
other side is pinned by a derivation that shares nothing with that chain: the canonical algorithm
is run at 60 digits with a relative perturbation delta_k injected after every operation (the model
of App. A.1: fl(a op b) = (a op b)(1 + delta), |delta| <= u; c u for an intrinsic with a c u
contract), and the first-order worst case sum_k |d y_i / d delta_k| c_k u is formed from central
differences.  A sound bound cannot be below it (up to second order), and the oracle's bound must
not exceed it by more than the looseness stated per template: the worst case over all summation
orders against the sequential one, absolute values where errors are correlated, a constant factor
where the template ignores a vanishing sensitivity.  The exact constants of these templates remain
"parity unpinned by the paper"; what these tests fix is that no term of them is missing and none is
over-estimated by the factors below."""
import mpmath as mp
import numpy as np
import pytest

mp.mp.dps = 60
U = mp.mpf(2) ** -24
f32 = np.float32


def _m(v):
    return mp.mpf(float(v))


def _first_order(fn, scales, nout):
    """sum_k |d out_i / d delta_k| scale_k u, by central differences at 60 digits."""
    h = mp.mpf(10) ** -25
    n = len(scales)
    tot = [mp.mpf(0)] * nout
    for k in range(n):
        dp = [mp.mpf(0)] * n
        dm = [mp.mpf(0)] * n
        dp[k], dm[k] = h, -h
        yp, ym = fn(dp), fn(dm)
        for i in range(nout):
            tot[i] += abs((yp[i] - ym[i]) / (2 * h)) * scales[k] * U
    return tot


def _layernorm(x, g, b, eps):
    n = len(x)

    def fn(d):
        it = iter(d)
        s = x[0]
        for i in range(1, n):
            s = (s + x[i]) * (1 + next(it))
        mu = (s / n) * (1 + next(it))
        dd = [(x[i] - mu) * (1 + next(it)) for i in range(n)]
        q = [(dd[i] * dd[i]) * (1 + next(it)) for i in range(n)]
        t = q[0]
        for i in range(1, n):
            t = (t + q[i]) * (1 + next(it))
        v = (t / n) * (1 + next(it))
        w = (v + eps) * (1 + next(it))
        r = (1 / mp.sqrt(w)) * (1 + next(it))
        hh = [(dd[i] * r) * (1 + next(it)) for i in range(n)]
        p = [(hh[i] * g[i]) * (1 + next(it)) for i in range(n)]
        return [(p[i] + b[i]) * (1 + next(it)) for i in range(n)]
    # c_div = 2 for the two divisions by n, c_rsqrt = 2 for the reciprocal square root
    scales = [1] * (n - 1) + [2] + [1] * n + [1] * n + [1] * (n - 1) + [2] + [1] + [2] + [1] * (3 * n)
    return fn, scales


def _rmsnorm(x, g, eps):
    n = len(x)

    def fn(d):
        it = iter(d)
        q = [(x[i] * x[i]) * (1 + next(it)) for i in range(n)]
        t = q[0]
        for i in range(1, n):
            t = (t + q[i]) * (1 + next(it))
        v = (t / n) * (1 + next(it))
        w = (v + eps) * (1 + next(it))
        r = (1 / mp.sqrt(w)) * (1 + next(it))
        hh = [(x[i] * r) * (1 + next(it)) for i in range(n)]
        return [(hh[i] * g[i]) * (1 + next(it)) for i in range(n)]
    scales = [1] * n + [1] * (n - 1) + [2] + [1] + [2] + [1] * (2 * n)
    return fn, scales


@pytest.mark.parametrize("n,median_max,worst_max", [(2, 1.42, 2.1), (3, 1.48, 2.1), (4, 1.56, 3.2)])
def test_layernorm_bound_is_within_a_stated_factor_of_the_first_order_worst_case(oracle_mod, n, median_max, worst_max):
    """Looseness: errors of the mean reach every output through d_i and through the variance, with signs
    that partly cancel, and the template adds their magnitudes: over random rows the ratio has a median of
    1.38 / 1.45 / 1.53 for 2 / 3 / 4 columns and stays below 2 / 2.2 / 3 (rows with an element near the
    mean).  The inputs are seeded, so the thresholds sit 3 % above what the template gives: a term of the chain
    over-estimated twofold moves the median by 8 % (the smallest of them) to 30 %."""
    rng = np.random.Generator(np.random.Philox(1000 + n))
    seen = []
    for trial in range(40):
        x = (rng.standard_normal(n) * (1 + trial % 6)).astype(f32)
        g = (1 + 0.3 * rng.standard_normal(n)).astype(f32)
        b = (0.5 * rng.standard_normal(n)).astype(f32)
        eps = 1e-5
        fn, scales = _layernorm([_m(v) for v in x], [_m(v) for v in g], [_m(v) for v in b], _m(f32(eps)))
        y = np.array([float(v) for v in fn([mp.mpf(0)] * len(scales))], f32)[None]
        fo = _first_order(fn, scales, n)
        tau = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x[None], y=y, g=g, b=b, eps=eps)[0]
        for i in range(n):
            ratio = _m(tau[i]) / fo[i]
            assert 1 - mp.mpf(10) ** -5 <= ratio <= worst_max, (n, trial, i, float(ratio))
            seen.append(float(ratio))
    print("median ratio", n, float(np.median(seen)), "max", max(seen))
    assert float(np.median(seen)) <= median_max, float(np.median(seen))


@pytest.mark.parametrize("n,loose", [(2, 1.02), (3, 1.06), (4, 1.12), (8, 1.35)])
def test_rmsnorm_bound_is_first_order_tight(oracle_mod, n, loose):
    """For two columns the template IS the first-order worst case (ratio 1.000); beyond, only the
    worst case over summation orders, Gamma(n-1), against the sequential sum's n-i separates them."""
    rng = np.random.Generator(np.random.Philox(50 + n))
    for trial in range(6):
        x = (rng.standard_normal(n) * (1 + trial)).astype(f32)
        g = (1 + 0.3 * rng.standard_normal(n)).astype(f32)
        eps = 1e-6
        fn, scales = _rmsnorm([_m(v) for v in x], [_m(v) for v in g], _m(f32(eps)))
        y = np.array([float(v) for v in fn([mp.mpf(0)] * len(scales))], f32)[None]
        fo = _first_order(fn, scales, n)
        tau = oracle_mod.bound_norm(oracle_mod.RMSNORM, x[None], y=y, g=g, eps=eps)[0]
        for i in range(n):
            if fo[i] == 0:
                continue
            ratio = _m(tau[i]) / fo[i]
            assert 1 - mp.mpf(10) ** -5 <= ratio <= loose, (n, trial, i, float(ratio))


def test_gelu_and_silu_bounds_against_the_first_order_worst_case(oracle_mod):
    """GELU (erf form): t = fl(x kappa), erf within c_erf u, fl(1 + erf), fl(0.5 x . ): ratio 1.00 - 1.34 (the
    template bounds |erf| by min(1, (2/sqrt(pi))|t|)).  SiLU: exp within c_exp u, fl(1 + e), fl(x / D): the
    template charges the exponential's error at full weight, although its sensitivity e/(1 + e) vanishes
    for large x: ratio 1.0 - 2.0 by construction."""
    o = oracle_mod
    kap = _m(f32(0.7071067811865476))
    worst_g, best_g, worst_s, best_s = 0.0, 10.0, 0.0, 10.0
    for xv in np.linspace(-4, 4, 41).astype(f32):
        if xv == 0:
            continue
        x = _m(xv)

        def gelu(d):
            t = (x * kap) * (1 + d[0])
            e = mp.erf(t) * (1 + d[1])
            s = (1 + e) * (1 + d[2])
            return [(x / 2 * s) * (1 + d[3])]
        y = np.array([float(gelu([mp.mpf(0)] * 4)[0])], f32)
        fo = _first_order(gelu, [1, 2, 1, 1], 1)[0]
        r = float(_m(o.bound_act(o.GELU_ERF, np.array([xv], f32), y)[0]) / fo)
        worst_g, best_g = max(worst_g, r), min(best_g, r)
    for xv in np.linspace(-8, 8, 41).astype(f32):
        if xv == 0:
            continue
        x = _m(xv)

        def silu(d):
            e = mp.e ** (-x) * (1 + d[0])
            D = (1 + e) * (1 + d[1])
            return [(x / D) * (1 + d[2])]
        y = np.array([float(silu([mp.mpf(0)] * 3)[0])], f32)
        fo = _first_order(silu, [2, 1, 1], 1)[0]
        r = float(_m(o.bound_act(o.SILU, np.array([xv], f32), y)[0]) / fo)
        worst_s, best_s = max(worst_s, r), min(best_s, r)
    assert 1 - 1e-5 <= best_g <= 1.01 and worst_g <= 1.4, (best_g, worst_g)
    assert 1 - 1e-5 <= best_s <= 1.01 and worst_s <= 2.0 + 1e-3, (best_s, worst_s)


def test_gelu_tanh_bound_against_the_first_order_worst_case(oracle_mod):
    """GELU, tanh form: p = sqrt(2/pi)(x + 0.044715 x^3) through seven roundings (five operations, the two
    constants), tanh within c_tanh u, fl(1 + tanh), fl(0.5 x . ).  The template charges all seven roundings
    on |p| although the cubic term carries four of them at a small weight for small |x|, and bounds |tanh|
    by min(1, |p|): ratio 1.00 - 1.51."""
    o = oracle_mod
    kap, c3 = mp.sqrt(2 / mp.pi), mp.mpf("0.044715")
    worst, best = 0.0, 10.0
    for xv in np.linspace(-5, 5, 51).astype(f32):
        if xv == 0:
            continue
        x = _m(xv)

        def gelu(d):
            k, c = kap * (1 + d[0]), c3 * (1 + d[1])
            x2 = (x * x) * (1 + d[2])
            x3 = (x2 * x) * (1 + d[3])
            t = (c * x3) * (1 + d[4])
            s = (x + t) * (1 + d[5])
            p = (k * s) * (1 + d[6])
            th = mp.tanh(p) * (1 + d[7])
            return [(x / 2 * ((1 + th) * (1 + d[8]))) * (1 + d[9])]
        y = np.array([float(gelu([mp.mpf(0)] * 10)[0])], f32)
        fo = _first_order(gelu, [1, 1, 1, 1, 1, 1, 1, 4, 1, 1], 1)[0]
        r = float(_m(o.bound_act(o.GELU_TANH, np.array([xv], f32), y)[0]) / fo)
        worst, best = max(worst, r), min(best, r)
    assert 1 - 1e-5 <= best <= 1.01 and worst <= 1.56, (best, worst)
