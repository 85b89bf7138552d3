"""Pins for the oracle's 2-D convolution bound (Sec. 3.1: conv is a reduction that takes
gamma_k with the k of the output element).  The direct triple loop is held against the exact
rational value of the definition, against an explicit patch matrix fed to the (separately
pinned) matmul bound, against closed forms with and without padding, and against real binary32
convolutions evaluated in several orders."""
from fractions import Fraction

import numpy as np
import pytest

from exact import f32_round, frac, up32


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _patches(x, R, S, stride, pad, dil):
    """Explicit patch matrix [Nb*OH*OW, R*S*C] of a channels-last tensor, zeros in the padding,
    columns ordered (r, s, c)."""
    Nb, H, W, C = x.shape
    OH = (H + 2 * pad[0] - dil[0] * (R - 1) - 1) // stride[0] + 1
    OW = (W + 2 * pad[1] - dil[1] * (S - 1) - 1) // stride[1] + 1
    out = np.zeros((Nb, OH, OW, R, S, C), x.dtype)
    for oh in range(OH):
        for ow in range(OW):
            for r in range(R):
                for s in range(S):
                    ih = oh * stride[0] - pad[0] + r * dil[0]
                    iw = ow * stride[1] - pad[1] + s * dil[1]
                    if 0 <= ih < H and 0 <= iw < W:
                        out[:, oh, ow, r, s, :] = x[:, ih, iw, :]
    return out.reshape(Nb * OH * OW, R * S * C), (Nb, OH, OW)


GEOMETRIES = [
    # Nb, H, W, C, Cout, R, S, stride, pad, dil, bias
    (1, 5, 6, 3, 4, 3, 3, (1, 1), (1, 1), (1, 1), True),
    (2, 7, 5, 2, 3, 3, 2, (2, 1), (0, 1), (1, 1), False),
    (1, 9, 8, 4, 2, 3, 3, (2, 2), (2, 2), (2, 2), True),
    (2, 4, 4, 5, 6, 1, 1, (1, 1), (0, 0), (1, 1), False),
    (1, 6, 7, 1, 2, 5, 3, (1, 2), (2, 0), (1, 2), True),
]


@pytest.mark.parametrize("geom", GEOMETRIES)
def test_conv_equals_matmul_bound_of_the_patch_matrix(oracle_mod, geom):
    Nb, H, W, C, Cout, R, S, stride, pad, dil, with_bias = geom
    rng = _rng(sum(geom[:7]))
    x = rng.standard_normal((Nb, H, W, C)).astype(np.float32)
    w = rng.standard_normal((Cout, R, S, C)).astype(np.float32)
    b = rng.standard_normal(Cout).astype(np.float32) if with_bias else None
    tau = oracle_mod.bound_conv2d(x, w, b, stride, pad, dil)
    P, (n, oh, ow) = _patches(x, R, S, stride, pad, dil)
    assert tau.shape == (n, oh, ow, Cout)
    want = oracle_mod.bound_linear(P, w.reshape(Cout, -1), b)
    # same terms in the same order (zeros add exactly): identical bits
    assert np.array_equal(tau.reshape(-1, Cout), want)


def test_conv_value_against_exact_rationals(oracle_mod):
    Nb, H, W, C, Cout, R, S = 1, 4, 5, 2, 3, 3, 3
    stride, pad, dil = (1, 2), (1, 1), (1, 1)
    rng = _rng(41)
    x = rng.standard_normal((Nb, H, W, C)).astype(np.float32)
    w = rng.standard_normal((Cout, R, S, C)).astype(np.float32)
    b = rng.standard_normal(Cout).astype(np.float32)
    tau = oracle_mod.bound_conv2d(x, w, b, stride, pad, dil)
    Kp = R * S * C + 1
    g = Fraction(Kp, 2 ** 24) / (1 - Fraction(Kp, 2 ** 24))
    OH, OW = tau.shape[1:3]
    assert (OH, OW) == (4, 3)
    for oh in range(OH):
        for ow in range(OW):
            for co in range(Cout):
                Ssum = abs(frac(b[co]))
                for r in range(R):
                    for s in range(S):
                        ih, iw = oh * stride[0] - pad[0] + r, ow * stride[1] - pad[1] + s
                        if 0 <= ih < H and 0 <= iw < W:
                            for c in range(C):
                                Ssum += abs(frac(x[0, ih, iw, c])) * abs(frac(w[co, r, s, c]))
                want = up32(g * Ssum)
                got = tau[0, oh, ow, co]
                assert got in (want, np.nextafter(want, np.float32(np.inf)))
                assert frac(got) >= g * Ssum


def test_conv_all_ones_closed_form_counts_valid_taps_but_keeps_full_k(oracle_mod):
    C, Cout = 8, 2
    x = np.ones((1, 5, 5, C), np.float32)
    w = np.ones((Cout, 3, 3, C), np.float32)
    K = 9 * C
    g = Fraction(K, 2 ** 24) / (1 - Fraction(K, 2 ** 24))
    t = oracle_mod.bound_conv2d(x, w, None, (1, 1), (1, 1), (1, 1))
    assert t.shape == (1, 5, 5, Cout)
    assert np.all(t[0, 1:4, 1:4] == up32(g * 9 * C))          # interior: nine taps
    assert np.all(t[0, 0, 1:4] == up32(g * 6 * C))            # edge: six taps, k still 9 C
    assert np.all(t[0, 0, 0] == up32(g * 4 * C)) and np.all(t[0, 4, 4] == up32(g * 4 * C))
    # no padding: 3 x 3 outputs, all interior
    t = oracle_mod.bound_conv2d(x, w, None)
    assert t.shape == (1, 3, 3, Cout) and np.all(t == up32(g * 9 * C))
    # with a bias the constant moves to k = K + 1 and |b| joins the sum
    b = np.full(Cout, -2.0, np.float32)
    g1 = Fraction(K + 1, 2 ** 24) / (1 - Fraction(K + 1, 2 ** 24))
    assert np.all(oracle_mod.bound_conv2d(x, w, b) == up32(g1 * (9 * C + 2)))


def test_conv_1x1_is_the_linear_bound_and_stride_subsamples(oracle_mod):
    rng = _rng(43)
    x = rng.standard_normal((2, 6, 7, 5)).astype(np.float32)
    w = rng.standard_normal((4, 1, 1, 5)).astype(np.float32)
    t = oracle_mod.bound_conv2d(x, w)
    assert np.array_equal(t.reshape(-1, 4), oracle_mod.bound_linear(x.reshape(-1, 5), w.reshape(4, 5)))
    w3 = rng.standard_normal((3, 3, 3, 5)).astype(np.float32)
    full = oracle_mod.bound_conv2d(x, w3, None, (1, 1), (1, 1))
    sub = oracle_mod.bound_conv2d(x, w3, None, (2, 3), (1, 1))
    assert np.array_equal(sub, full[:, ::2, ::3])
    # sign-blind in both operands, homogeneous for powers of two
    assert np.array_equal(oracle_mod.bound_conv2d(-x, np.abs(w3), None, (1, 1), (1, 1)), full)
    assert np.array_equal(oracle_mod.bound_conv2d(x * np.float32(4), w3, None, (1, 1), (1, 1)), full * np.float32(4))


def test_conv_bound_is_sound_for_real_binary32_convolutions(oracle_mod):
    """|computed - exact| <= tau for binary32 convolutions accumulated in several orders
    (forward, reversed, pairwise, fused multiply-add chain), exact value from rationals."""
    rng = _rng(44)
    Nb, H, W, C, Cout, R, S = 1, 4, 4, 3, 2, 3, 3
    worst = 0.0
    for trial in range(6):
        x = (rng.standard_normal((Nb, H, W, C)) * 2.0 ** rng.integers(-6, 7)).astype(np.float32)
        w = rng.standard_normal((Cout, R, S, C)).astype(np.float32)
        b = rng.standard_normal(Cout).astype(np.float32)
        tau = oracle_mod.bound_conv2d(x, w, b, (1, 1), (1, 1))
        P, _ = _patches(x, R, S, (1, 1), (1, 1), (1, 1))
        Wm = w.reshape(Cout, -1)
        for i in range(P.shape[0]):
            for co in range(Cout):
                a, v = P[i], Wm[co]
                exact = sum(frac(p) * frac(q) for p, q in zip(a, v)) + frac(b[co])
                prods = [np.float32(p * q) for p, q in zip(a, v)]
                results = []
                acc = np.float32(0)
                for p in prods: acc = np.float32(acc + p)
                results.append(np.float32(acc + b[co]))
                acc = b[co]
                for p in reversed(prods): acc = np.float32(acc + p)
                results.append(acc)
                items = prods + [b[co]]
                while len(items) > 1:
                    items = [np.float32(items[k] + items[k + 1]) if k + 1 < len(items) else items[k]
                             for k in range(0, len(items), 2)]
                results.append(items[0])
                accq = frac(b[co])
                for p, q in zip(a, v): accq = frac(f32_round(accq + frac(p) * frac(q)))
                results.append(float(accq))
                t = frac(tau.reshape(-1, Cout)[i, co])
                for r in results:
                    err = abs(Fraction(float(r)) - exact)
                    assert err <= t
                    if t > 0: worst = max(worst, float(err / t))
    assert 0.0 < worst <= 1.0


def test_conv_rejects_bad_geometry(oracle_mod):
    x = np.zeros((1, 2, 2, 1), np.float32)
    w = np.zeros((1, 3, 3, 1), np.float32)
    with pytest.raises(ValueError):
        oracle_mod.bound_conv2d(x, w)                    # filter larger than the unpadded input
    with pytest.raises(ValueError):
        oracle_mod.bound_conv2d(x, w, None, (0, 1), (1, 1))
