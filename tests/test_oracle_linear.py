"""Pins for the oracle's linear/matmul and sum/mean bounds (Sec. 3.1 reductions;
App. A.2 Eq. det-sum): exact-rational brute force over every summation order,
closed forms, homogeneity, monotonicity, operand layout."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from exact import all_fp32_sums, f32_round, frac, up32


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _dot_results(a, w, bias):
    """All binary32 results of sum_k a_k w_k (+ bias): products rounded separately, any
    addition order; plus the sequential fused-multiply-add chains in every order."""
    prods = [np.float32(x * y) for x, y in zip(a, w)]
    terms = prods + ([np.float32(bias)] if bias is not None else [])
    res = set(all_fp32_sums(terms))
    K = len(a)
    for perm in itertools.permutations(range(K)):
        for bias_first in ((True, False) if bias is not None else (False,)):
            acc = frac(bias) if (bias is not None and bias_first) else Fraction(0)
            for k in perm:
                acc = frac(f32_round(acc + frac(a[k]) * frac(w[k])))
            if bias is not None and not bias_first:
                acc = frac(f32_round(acc + frac(bias)))
            res.add(float(acc))
    return res


@pytest.mark.parametrize("K,with_bias", [(1, False), (2, False), (3, True), (4, False), (4, True)])
def test_linear_bound_is_sound_for_every_order(oracle_mod, K, with_bias):
    rng = _rng(100 + K + 10 * with_bias)
    worst = 0.0
    for trial in range(25):
        scale = np.float32(2.0 ** rng.integers(-8, 9))
        a = (rng.standard_normal(K).astype(np.float32) * scale)
        w = rng.standard_normal(K).astype(np.float32)
        b = np.float32(rng.standard_normal()) if with_bias else None
        exact = sum(frac(x) * frac(y) for x, y in zip(a, w)) + (frac(b) if with_bias else 0)
        tau = oracle_mod.bound_linear(a[None, :], w[None, :],
                                      None if b is None else np.array([b], np.float32))[0, 0]
        for r in _dot_results(a, w, b):
            err = abs(Fraction(r) - exact)
            assert err <= frac(tau), (a, w, b, r)
            if tau > 0:
                worst = max(worst, float(err / frac(tau)))
    assert worst > 0.0 or K == 1     # the test really exercised rounding


def test_linear_value_is_gamma_times_abs_product(oracle_mod):
    rng = _rng(7)
    for K, N, M, with_bias in ((5, 3, 4, False), (37, 6, 5, True), (256, 4, 3, True)):
        A = rng.standard_normal((M, K)).astype(np.float32)
        W = rng.standard_normal((N, K)).astype(np.float32)
        b = rng.standard_normal(N).astype(np.float32) if with_bias else None
        tau = oracle_mod.bound_linear(A, W, b)
        Kp = K + (1 if with_bias else 0)
        g = Fraction(Kp, 2 ** 24) / (1 - Fraction(Kp, 2 ** 24))
        for i in range(M):
            for j in range(N):
                S = sum(abs(frac(A[i, k])) * abs(frac(W[j, k])) for k in range(K))
                if with_bias:
                    S += abs(frac(b[j]))
                want = up32(g * S)
                # directed binary64 evaluation may sit a hair above the exact value
                assert tau[i, j] in (want, np.nextafter(want, np.float32(np.inf)))
                assert frac(tau[i, j]) >= g * S


def test_linear_all_ones_closed_form(oracle_mod):
    for K in (1, 16, 256, 2048):
        A = np.ones((2, K), np.float32)
        W = np.ones((3, K), np.float32)
        tau = oracle_mod.bound_linear(A, W)
        g = Fraction(K, 2 ** 24) / (1 - Fraction(K, 2 ** 24))
        assert np.all(tau == up32(K * g))


def test_linear_layout_transposed_and_batched(oracle_mod):
    rng = _rng(11)
    A = rng.standard_normal((2, 5, 9)).astype(np.float32)
    W = rng.standard_normal((2, 7, 9)).astype(np.float32)
    t0 = oracle_mod.bound_linear(A, W)
    t1 = oracle_mod.bound_linear(A, np.ascontiguousarray(W.transpose(0, 2, 1)), trans_w=True)
    assert t0.shape == (2, 5, 7)
    assert np.array_equal(t0, t1)
    for b in range(2):
        assert np.array_equal(t0[b], oracle_mod.bound_linear(A[b], W[b]))
    # rows of A index rows of tau, rows of W index columns of tau
    A2 = A[0].copy(); A2[3] = 0
    assert np.all(oracle_mod.bound_linear(A2, W[0])[3] == 0)
    W2 = W[0].copy(); W2[4] = 0
    assert np.all(oracle_mod.bound_linear(A[0], W2)[:, 4] == 0)


def test_linear_homogeneous_sign_blind_monotone(oracle_mod):
    rng = _rng(12)
    A = rng.standard_normal((4, 33)).astype(np.float32)
    W = rng.standard_normal((6, 33)).astype(np.float32)
    t = oracle_mod.bound_linear(A, W)
    assert np.array_equal(oracle_mod.bound_linear(A * np.float32(8), W), t * np.float32(8))
    assert np.array_equal(oracle_mod.bound_linear(-A, W), t)
    assert np.array_equal(oracle_mod.bound_linear(A, -np.abs(W)), t)
    # appending zero columns raises K and therefore the bound
    Az = np.concatenate([A, np.zeros((4, 31), np.float32)], axis=1)
    Wz = np.concatenate([W, np.zeros((6, 31), np.float32)], axis=1)
    assert np.all(oracle_mod.bound_linear(Az, Wz) > t)
    # probabilistic mode is tighter at K = 64
    assert np.all(oracle_mod.bound_linear(Az, Wz, model=oracle_mod.Model(mode=1)) <
                  oracle_mod.bound_linear(Az, Wz))


def test_linear_k_out_of_range(oracle_mod):
    # K u >= 1: constant undefined (App. A.1), reported as a status
    A = np.zeros((1, 2 ** 24), np.float32)
    with pytest.raises(ValueError):
        oracle_mod.bound_linear(A, A)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
def test_sum_and_mean_sound_for_every_order(oracle_mod, n):
    rng = _rng(200 + n)
    for trial in range(8 if n >= 6 else 20):
        x = rng.standard_normal(n).astype(np.float32) * np.float32(2.0 ** rng.integers(-4, 5))
        exact = sum(frac(v) for v in x)
        tau_s = oracle_mod.bound_norm(oracle_mod.SUM, x[None, :])[0]
        sums = all_fp32_sums(list(x))
        for s in sums:
            assert abs(Fraction(s) - exact) <= frac(tau_s)
        if n == 1:
            assert tau_s == 0.0
        # mean: divide by n, or multiply by the rounded reciprocal (both within c_div = 2)
        for s in sums:
            s32 = np.float32(s)
            for y in (np.float32(s32 / np.float32(n)),
                      np.float32(s32 * np.float32(np.float32(1) / np.float32(n)))):
                tau_m = oracle_mod.bound_norm(oracle_mod.MEAN, x[None, :],
                                              y=np.array([y], np.float32))[0]
                assert abs(frac(y) - exact / n) <= frac(tau_m)


def test_sum_closed_form(oracle_mod):
    n = 257
    x = -np.ones((1, n), np.float32)
    g = Fraction(n - 1, 2 ** 24) / (1 - Fraction(n - 1, 2 ** 24))
    assert oracle_mod.bound_norm(oracle_mod.SUM, x)[0] == up32(g * n)
    y = np.array([-1.0], np.float32)
    cu = Fraction(2, 2 ** 24)
    want = g + cu / (1 - cu)
    got = oracle_mod.bound_norm(oracle_mod.MEAN, x, y=y)[0]
    assert frac(got) >= want and frac(np.nextafter(got, np.float32(0))) <= want * (1 + Fraction(1, 2 ** 40))
