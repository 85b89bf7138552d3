"""Pins for the oracle's LayerNorm / RMSNorm / BatchNorm-affine bounds (operators
named in App. A.3; templates derived from the primitive rule of Sec. 3.1):
brute-force soundness of binary32 canonical executions against 60-digit values,
closed form on a constant row, equivariance, failure rows."""
import itertools
from fractions import Fraction

import mpmath as mp
import numpy as np
import pytest

from exact import all_fp32_sums, f32_round, frac

mp.mp.dps = 60
U = 2.0 ** -24
f32 = np.float32


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _mpf(v):
    return mp.mpf(float(v))


def _to_frac(m):
    m = mp.mpf(m)
    v = Fraction(int(m.man)) * (Fraction(2) ** int(m.exp))
    return -v if m._mpf_[0] else v


def _pick(values, rng, k=4):
    vals = sorted(values)
    if len(vals) <= k:
        return [f32(v) for v in vals]
    idx = {0, len(vals) - 1} | set(rng.integers(0, len(vals), k - 2).tolist())
    return [f32(vals[i]) for i in sorted(idx)]


def _div_n(s, n):
    """Both ways a kernel may divide by n."""
    return [f32(s / f32(n)), f32(s * f32(f32(1) / f32(n)))]


def _rsqrt_variants(w, rng, c=2.0):
    exact = 1 / mp.sqrt(_mpf(w))
    out = [f32_round(_to_frac(exact * (1 + mp.mpf((c - 1) * U * 0.99 * rng.uniform(-1, 1)))))]
    out.append(f32(f32(1) / f32(np.sqrt(f32(w)))))          # sqrt then divide: two roundings
    return out


def _layernorm_runs(x, g, b, eps, rng):
    n = len(x)
    eps32 = f32(eps)
    for s in _pick(all_fp32_sums(list(x)), rng):
        for mu in _div_n(s, n):
            d = [f32(v - mu) for v in x]
            q = [f32(v * v) for v in d]
            for t in _pick(all_fp32_sums(q), rng):
                for v in _div_n(t, n):
                    w = f32(v + eps32)
                    for r in _rsqrt_variants(w, rng):
                        h = [f32(dd * r) for dd in d]
                        p = [f32(hh * gg) for hh, gg in zip(h, g)]
                        yield np.array([f32(pp + bb) for pp, bb in zip(p, b)], f32)


def _layernorm_exact(x, g, b, eps):
    n = len(x)
    xs = [_mpf(v) for v in x]
    mu = mp.fsum(xs) / n
    d = [v - mu for v in xs]
    var = mp.fsum([v * v for v in d]) / n
    r = 1 / mp.sqrt(var + _mpf(f32(eps)))
    return [dd * r * _mpf(gg) + _mpf(bb) for dd, gg, bb in zip(d, g, b)]


@pytest.mark.parametrize("n", [2, 3, 4, 5])
def test_layernorm_bound_is_sound(oracle_mod, n):
    rng = _rng(500 + n)
    runs = 0
    for trial in range(6):
        x = (rng.standard_normal(n) * rng.choice([1.0, 30.0]) + rng.choice([0.0, 5.0])).astype(f32)
        g = (rng.standard_normal(n) + 1).astype(f32)
        b = rng.standard_normal(n).astype(f32)
        eps = float(rng.choice([1e-5, 1e-12]))
        ystar = _layernorm_exact(x, g, b, eps)
        for y in _layernorm_runs(x, g, b, eps, rng):
            tau = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x[None], y=y[None], g=g, b=b, eps=eps)[0]
            runs += 1
            for i in range(n):
                assert abs(_mpf(y[i]) - ystar[i]) <= _mpf(tau[i]), (x, g, b, eps, y, i)
            # without the re-executed output the fresh-rounding term is taken at an upper bound of
            # |y| over all canonical executions: never below the bound that knows y
            tau0 = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x[None], y=None, g=g, b=b, eps=eps)[0]
            assert np.all(tau0 >= tau)
            # not absurdly loose: a few hundred u relative to the scale of the output
            scale = np.abs(g).max() * np.sqrt(n) + np.abs(b).max()
            assert np.all(tau < 2000 * U * scale)
    assert runs >= 40


def test_layernorm_constant_row_closed_form(oracle_mod):
    n, c, eps = 16, 1.0, 1e-5
    x = np.full((1, n), c, f32)
    g = np.linspace(0.5, 2.0, n).astype(f32)
    b = np.linspace(-1, 1, n).astype(f32)
    y = b[None].copy()                       # d = 0 exactly, so y = b
    tau = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x, y=y, g=g, b=b, eps=eps)[0]
    u = mp.mpf(2) ** -24
    G = (n - 1) * u / (1 - (n - 1) * u)
    cu = 2 * u
    E_s = G * n * c
    E_mu = (E_s / n + cu * c) / (1 - cu)
    E_d = E_mu / (1 - u)
    D = E_d
    E_q = E_d * D + u * D * D
    Q = D * D * (1 + u)
    E_t = G * n * Q + n * E_q
    E_v = (E_t / n) / (1 - cu)
    eps32 = _mpf(f32(eps))
    E_w = (E_v + u * eps32) / (1 - u)
    w_lo = eps32 - E_w
    E_r = E_w / 2 * w_lo ** mp.mpf(-1.5) + 2 * u * w_lo ** mp.mpf(-0.5)
    rs = eps32 ** mp.mpf(-0.5)
    R = rs + E_r
    E_h = D * E_r + rs * E_d + u * D * R
    for i in range(n):
        ag = abs(_mpf(g[i]))
        want = ag * E_h + u * ag * E_h + u * abs(_mpf(b[i]))
        got = _mpf(tau[i])
        assert want <= got <= want * (1 + mp.mpf(2) ** -22)


def test_layernorm_no_finite_bound_gives_nan(oracle_mod):
    # constant row with a tiny eps: the lower end of v + eps is not positive
    x = np.full((2, 8), 3.0, f32); x[1] = np.arange(8)
    y = np.zeros((2, 8), f32)
    tau = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x, y=y, eps=1e-12)
    assert np.all(np.isnan(tau[0])) and np.all(np.isfinite(tau[1]))


def test_layernorm_equivariance(oracle_mod):
    rng = _rng(9)
    n = 48
    x = rng.standard_normal((3, n)).astype(f32)
    g = rng.standard_normal(n).astype(f32)
    xd = x.astype(np.float64)
    y = ((xd - xd.mean(1, keepdims=True)) / np.sqrt(xd.var(1, keepdims=True) + 1e-5) * g).astype(f32)
    t = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x, y=y, g=g, eps=1e-5)
    t2 = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x, y=y * f32(4), g=g * f32(4), eps=1e-5)
    assert np.array_equal(t2, t * f32(4))
    p = rng.permutation(n)
    tp = oracle_mod.bound_norm(oracle_mod.LAYERNORM, x[:, p], y=y[:, p], g=g[p], eps=1e-5)
    assert np.allclose(tp, t[:, p], rtol=1e-6, atol=0)       # sums are re-associated
    # g = None means g = 1
    y1 = ((xd - xd.mean(1, keepdims=True)) / np.sqrt(xd.var(1, keepdims=True) + 1e-5)).astype(f32)
    assert np.array_equal(oracle_mod.bound_norm(oracle_mod.LAYERNORM, x, y=y1, eps=1e-5),
                          oracle_mod.bound_norm(oracle_mod.LAYERNORM, x, y=y1, g=np.ones(n, f32), eps=1e-5))


def _rmsnorm_runs(x, g, eps, rng):
    n = len(x)
    q = [f32(v * v) for v in x]
    for t in _pick(all_fp32_sums(q), rng, 6):
        for v in _div_n(t, n):
            w = f32(v + f32(eps))
            for r in _rsqrt_variants(w, rng):
                yield np.array([f32(gg * f32(xx * r)) for xx, gg in zip(x, g)], f32)


@pytest.mark.parametrize("n", [1, 2, 4, 6])
def test_rmsnorm_bound_is_sound(oracle_mod, n):
    rng = _rng(600 + n)
    for trial in range(8):
        x = (rng.standard_normal(n) * rng.choice([0.01, 1.0, 100.0])).astype(f32)
        g = (rng.standard_normal(n) + 1).astype(f32)
        eps = 1e-6
        xs = [_mpf(v) for v in x]
        r = 1 / mp.sqrt(mp.fsum([v * v for v in xs]) / n + _mpf(f32(eps)))
        ystar = [xx * r * _mpf(gg) for xx, gg in zip(xs, g)]
        for y in _rmsnorm_runs(x, g, eps, rng):
            tau = oracle_mod.bound_norm(oracle_mod.RMSNORM, x[None], y=y[None], g=g, eps=eps)[0]
            for i in range(n):
                assert abs(_mpf(y[i]) - ystar[i]) <= _mpf(tau[i])
            assert np.all(tau <= (n + 12) * 2 * U * np.abs(y) + 1e-30)
            tau0 = oracle_mod.bound_norm(oracle_mod.RMSNORM, x[None], y=None, g=g, eps=eps)[0]
            assert np.all(tau0 >= tau) and np.all(tau0 <= tau * (1 + 8 * U) + 1e-30)


def test_rmsnorm_constant_magnitude_closed_form(oracle_mod):
    n, c, eps = 64, 0.75, 1e-6
    rng = _rng(10)
    x = (c * rng.choice([-1.0, 1.0], n)).astype(f32)[None]
    g = np.ones(n, f32)
    eps32 = _mpf(f32(eps))
    rs = 1 / mp.sqrt(mp.mpf(c) ** 2 + eps32)
    y = np.array([f32(float(v * rs)) for v in x[0]], f32)[None]
    tau = oracle_mod.bound_norm(oracle_mod.RMSNORM, x, y=y, g=g, eps=eps)[0]
    u = mp.mpf(2) ** -24
    G = (n - 1) * u / (1 - (n - 1) * u)
    cu = 2 * u
    v = mp.mpf(c) ** 2
    E_t = (G * (1 + u) + u) * n * v
    E_v = (E_t / n + cu * v) / (1 - cu)
    E_w = (E_v + u * (v + eps32)) / (1 - u)
    w_lo = v + eps32 - E_w
    E_r = E_w / 2 * w_lo ** mp.mpf(-1.5) + 2 * u * w_lo ** mp.mpf(-0.5)
    R = rs + E_r
    for i in range(n):
        want = mp.mpf(c) * (E_r + u * R) + u * abs(_mpf(y[0, i]))
        assert want <= _mpf(tau[i]) <= want * (1 + mp.mpf(2) ** -22)
    # the same row without y: the fresh-rounding term at Y = |x g| R (1+u)^2
    tau0 = oracle_mod.bound_norm(oracle_mod.RMSNORM, x, y=None, g=g, eps=eps)[0]
    for i in range(n):
        want = mp.mpf(c) * (E_r + u * R) + u * mp.mpf(c) * R * (1 + u) ** 2
        assert want <= _mpf(tau0[i]) <= want * (1 + mp.mpf(2) ** -22)
    # first-order size: |y| (gamma_n/2 + (c_rsqrt + c_div/2 + 2.5) u), about (n/2 + 5.5) u |y|
    assert np.all(np.abs(tau / np.abs(y[0]) / U - (n / 2 + 5.5)) < 1.0)


def test_bn_affine_sound_fused_and_unfused(oracle_mod):
    rng = _rng(11)
    C = 7
    x = np.abs(rng.standard_normal((5, C))).astype(f32)
    s = (rng.standard_normal(C) * 2).astype(f32)
    t = rng.standard_normal(C).astype(f32)
    for fused in (False, True):
        y = np.empty_like(x)
        for i in range(5):
            for c in range(C):
                if fused:
                    y[i, c] = f32_round(frac(x[i, c]) * frac(s[c]) + frac(t[c]))
                else:
                    y[i, c] = f32(f32(x[i, c] * s[c]) + t[c])
        tau = oracle_mod.bound_norm(oracle_mod.BN_AFFINE, x, y=y, g=s, b=t)
        for i in range(5):
            for c in range(C):
                exact = frac(x[i, c]) * frac(s[c]) + frac(t[c])
                assert abs(frac(y[i, c]) - exact) <= frac(tau[i, c])
                want = Fraction(1, 2 ** 24) * abs(frac(x[i, c]) * frac(s[c])) * (1 + Fraction(1, 2 ** 24)) \
                    + Fraction(1, 2 ** 24) * abs(frac(y[i, c]))
                assert want <= frac(tau[i, c]) <= want * (1 + Fraction(1, 2 ** 22))


def test_bounds_without_the_reexecuted_output(oracle_mod):
    """y = None: the term u|y| of the primitive rule (Sec. 3.1) is evaluated at an upper bound Y of
    |y| built from exact intermediates: closed forms in exact rationals (BatchNorm-affine, mean) and
    against 60-digit intermediates (LayerNorm)."""
    rng = _rng(77)
    u = Fraction(1, 2 ** 24)
    C = 9
    x = rng.standard_normal((4, C)).astype(f32)
    s = (rng.standard_normal(C) * 2).astype(f32)
    t = rng.standard_normal(C).astype(f32)
    for shift in (t, None):
        tau = oracle_mod.bound_norm(oracle_mod.BN_AFFINE, x, y=None, g=s, b=shift)
        for i in range(4):
            for c in range(C):
                xs = abs(frac(x[i, c]) * frac(s[c]))
                at = abs(frac(shift[c])) if shift is not None else 0
                want = u * xs * (1 + u) + u * (xs * (1 + u) + at) * (1 + u)
                assert want <= frac(tau[i, c]) <= want * (1 + Fraction(1, 2 ** 22))
    # mean of n terms: Gamma(n-1) sum|x| / n + Y c u/(1 - c u), Y = (sum|x|/n)(1 + Gamma(n-1))(1 + c u), c = c_div = 2
    for n in (1, 3, 17):
        xr = rng.standard_normal((2, n)).astype(f32)
        tau = oracle_mod.bound_norm(oracle_mod.MEAN, xr, y=None)
        for r in range(2):
            sa = sum(abs(frac(v)) for v in xr[r])
            G = (n - 1) * u / (1 - (n - 1) * u)
            cu = 2 * u
            want = G * sa / n + (sa / n) * (1 + G) * (1 + cu) * cu / (1 - cu)
            assert want <= frac(tau[r]) <= want * (1 + Fraction(1, 2 ** 22)) + Fraction(1, 2 ** 149)
            # and it covers the bound of any actual mean
            y = np.array([f32(np.sum(xr[r], dtype=f32) / f32(n))], f32)
            assert tau[r] >= oracle_mod.bound_norm(oracle_mod.MEAN, xr[r:r + 1], y=y)[0]
    # LayerNorm: tau(None) = E_p + u (|d*| r* |g| + E_p + |b|)(1+u) with E_p = tau(y) - u|y| of the branch
    # pinned above and d*, r* from 60-digit arithmetic
    n = 12
    xl = (rng.standard_normal((3, n)) * 2 + 1).astype(f32)
    g = (rng.standard_normal(n) + 1).astype(f32)
    b = rng.standard_normal(n).astype(f32)
    eps = 1e-5
    um = mp.mpf(2) ** -24
    for use_b in (True, False):
        bb = b if use_b else None
        y = np.array([[f32(float(v)) for v in _layernorm_exact(row, g, b if use_b else np.zeros(n, f32), eps)] for row in xl], f32)
        t_y = oracle_mod.bound_norm(oracle_mod.LAYERNORM, xl, y=y, g=g, b=bb, eps=eps)
        t_0 = oracle_mod.bound_norm(oracle_mod.LAYERNORM, xl, y=None, g=g, b=bb, eps=eps)
        for r in range(3):
            xs = [_mpf(v) for v in xl[r]]
            mu = mp.fsum(xs) / n
            d = [v - mu for v in xs]
            rs = 1 / mp.sqrt(mp.fsum([v * v for v in d]) / n + _mpf(f32(eps)))
            for i in range(n):
                E_p = _mpf(t_y[r, i]) - um * abs(_mpf(y[r, i]))
                want = E_p + um * (abs(d[i]) * rs * abs(_mpf(g[i])) + E_p + (abs(_mpf(b[i])) if use_b else 0)) * (1 + um)
                assert want * (1 - mp.mpf(2) ** -22) <= _mpf(t_0[r, i]) <= want * (1 + mp.mpf(2) ** -21)
    # a planted mistake would show: leaving |b| out of Y changes the LayerNorm bound
    assert np.any(oracle_mod.bound_norm(oracle_mod.LAYERNORM, xl, y=None, g=g, b=b, eps=eps) >
                  oracle_mod.bound_norm(oracle_mod.LAYERNORM, xl, y=None, g=g, b=None, eps=eps))


# ---- GroupNorm (App. A.3 operator list): LayerNorm over each (sample, group) -------------------

def _groupnorm_two_pass(x, groups, g, b, eps, dtype):
    """The canonical two-pass algorithm on x[N, C, H, W] in the given precision."""
    N, C = x.shape[:2]
    xr = x.reshape(N, groups, -1).astype(dtype)
    n = xr.shape[-1]
    mu = (xr.sum(axis=-1, keepdims=True, dtype=dtype) / dtype(n)).astype(dtype)
    d = (xr - mu).astype(dtype)
    var = ((d * d).astype(dtype).sum(axis=-1, keepdims=True, dtype=dtype) / dtype(n)).astype(dtype)
    r = (dtype(1) / np.sqrt((var + dtype(np.float32(eps))).astype(dtype))).astype(dtype)
    h = (d * r).astype(dtype).reshape(x.shape)
    shape = (1, C) + (1,) * (x.ndim - 2)
    return ((h * g.reshape(shape).astype(dtype)).astype(dtype) + b.reshape(shape).astype(dtype)).astype(dtype)


def test_groupnorm_is_layernorm_per_group_with_repeated_affine(oracle_mod):
    o = oracle_mod
    rng = np.random.Generator(np.random.Philox(71))
    N, C, H, W, G = 3, 12, 4, 5, 4
    x = rng.standard_normal((N, C, H, W)).astype(f32)
    g = (1 + 0.3 * rng.standard_normal(C)).astype(f32); b = rng.standard_normal(C).astype(f32)
    y = _groupnorm_two_pass(x, G, g, b, 1e-5, f32)
    tau = o.bound_groupnorm(x, y, G, g, b, eps=1e-5)
    assert tau.shape == x.shape
    # one group, one position: plain LayerNorm over the channels
    x1 = x[:, :, 0, 0].copy(); y1 = _groupnorm_two_pass(x1[:, :, None, None], 1, g, b, 1e-5, f32)[:, :, 0, 0]
    assert np.array_equal(o.bound_groupnorm(x1[:, :, None, None], y1[:, :, None, None], 1, g, b, eps=1e-5)[:, :, 0, 0],
                          o.bound_norm(o.LAYERNORM, x1, y=y1, g=g, b=b, eps=1e-5))
    # a (sample, group) block on its own, element by element against the LayerNorm bound
    cpg = C // G
    for n_, j in ((0, 0), (2, 3), (1, 2)):
        row = x[n_, j * cpg:(j + 1) * cpg].reshape(1, -1)
        yrow = y[n_, j * cpg:(j + 1) * cpg].reshape(1, -1)
        want = o.bound_norm(o.LAYERNORM, row, y=yrow, g=np.repeat(g[j * cpg:(j + 1) * cpg], H * W),
                            b=np.repeat(b[j * cpg:(j + 1) * cpg], H * W), eps=1e-5)
        assert np.array_equal(tau[n_, j * cpg:(j + 1) * cpg].reshape(1, -1), want)
    # groups == channels is instance normalisation: every channel its own row, scalar affine
    ti = o.bound_groupnorm(x, _groupnorm_two_pass(x, C, g, b, 1e-5, f32), C, g, b, eps=1e-5)
    c = 7
    yi = _groupnorm_two_pass(x, C, g, b, 1e-5, f32)
    want = o.bound_norm(o.LAYERNORM, x[1, c].reshape(1, -1), y=yi[1, c].reshape(1, -1),
                        g=np.full(H * W, g[c], f32), b=np.full(H * W, b[c], f32), eps=1e-5)
    assert np.array_equal(ti[1, c].reshape(1, -1), want)
    with pytest.raises(ValueError):
        o.bound_groupnorm(x, y, 5, g, b)


def test_groupnorm_bound_is_sound_and_follows_channel_permutations(oracle_mod):
    o = oracle_mod
    rng = np.random.Generator(np.random.Philox(72))
    N, C, H, W, G = 2, 8, 6, 6, 2
    worst = 0.0
    for trial in range(5):
        x = (rng.standard_normal((N, C, H, W)) * 2.0 ** rng.integers(-4, 5) + rng.standard_normal()).astype(f32)
        g = (1 + 0.5 * rng.standard_normal(C)).astype(f32); b = rng.standard_normal(C).astype(f32)
        y = _groupnorm_two_pass(x, G, g, b, 1e-5, f32)
        ystar = _groupnorm_two_pass(x.astype(np.float64), G, g, b, 1e-5, np.float64)
        tau = o.bound_groupnorm(x, y, G, g, b, eps=1e-5)
        err = np.abs(y.astype(np.float64) - ystar)
        assert np.all(err <= tau.astype(np.float64) + 1e-13 * np.abs(ystar))
        worst = max(worst, float((err / tau).max()))
    assert 0.02 < worst <= 1.0
    # permuting the channels inside each group (with their affine parameters) permutes tau
    cpg = C // G
    perm = np.concatenate([j * cpg + rng.permutation(cpg) for j in range(G)])
    xp, yp = x[:, perm], y[:, perm]
    tp = o.bound_groupnorm(xp, yp, G, g[perm], b[perm], eps=1e-5)
    # the sums run over the same multiset in another order: equal up to the last bits of binary64
    assert np.all(np.abs(tp / tau[:, perm] - 1) < 1e-6)
