"""Pins for the oracle's leaf check (Sec. 5.4) and relative-error profile
(Sec. 5.3, Sec. 3.2 Eq. 2) on the fixed 2048-edge histogram: constructed cases
with known counts, bins and ranks; exact order statistics by sorting."""
import numpy as np
import pytest

f32 = np.float32


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _bin(v):
    return int(np.array([v], f32).view(np.uint32)[0] >> 20)


def test_constructed_errors_land_in_known_bins(oracle_mod):
    # claimed = ref (1 + 2^-k) exactly, eps = 0  =>  e = 2^-k exactly
    ref = np.array([1.0, -2.0, 0.5, 3.0, 1.0], f32)
    ks = [10, 12, 10, 20, 23]
    claimed = np.array([r * (1 + 2.0 ** -k) for r, k in zip(ref, ks)], f32)
    tau = np.abs(claimed.astype(np.float64) - ref).astype(f32)       # exact differences
    p = oracle_mod.check_and_profile(claimed, ref, tau, alpha=1.0, eps_rel=0.0)
    assert p["n"] == 5 and p["violations"] == 0 and p["accept"] == 1 and p["nan_count"] == 0
    for k in set(ks):
        assert p["hist"][(127 - k) << 3] == ks.count(k)
    assert p["hist"].sum() == 5
    assert p["max_rel"] == f32(2.0 ** -10)
    # shrink tau by one ulp on two elements: exactly those violate (the test is d <= tau)
    tau2 = tau.copy(); tau2[[1, 3]] = np.nextafter(tau2[[1, 3]], f32(0))
    q = oracle_mod.check_and_profile(claimed, ref, tau2, alpha=1.0, eps_rel=0.0)
    assert q["violations"] == 2 and q["accept"] == 0
    # alpha scales the bound (Sec. 4.5 scale factor): 2x loosens, 0.5x tightens
    assert oracle_mod.check_and_profile(claimed, ref, tau2, alpha=2.0, eps_rel=0.0)["violations"] == 0
    assert oracle_mod.check_and_profile(claimed, ref, tau, alpha=0.5, eps_rel=0.0)["violations"] == 5


def test_relative_error_uses_reference_magnitude_plus_eps(oracle_mod):
    ref = np.array([4.0, 0.0], f32)
    claimed = np.array([5.0, 0.25], f32)
    tau = np.ones(2, f32)
    p = oracle_mod.check_and_profile(claimed, ref, tau, eps_rel=0.5)
    e = np.sort(oracle_mod.rel_errors(claimed, ref, eps_rel=0.5))
    assert e[0] == f32(1.0 / 4.5) and e[1] == f32(0.5)
    assert p["hist"][_bin(f32(1.0 / 4.5))] == 1 and p["hist"][_bin(0.5)] == 1
    # swapping roles changes the denominator: it is |ref|, not |claimed|
    e2 = oracle_mod.rel_errors(ref, claimed, eps_rel=0.5)
    assert e2[0] == f32(1.0 / 5.5)


def test_nan_inf_and_zero_denominator(oracle_mod):
    ref = np.array([1.0, 0.0, 0.0, np.nan, 1.0, np.inf], f32)
    claimed = np.array([1.0, 0.0, 1.0, 1.0, np.nan, np.inf], f32)
    tau = np.array([0.0, 0.0, 2.0, 1.0, 1.0, 1.0], f32)
    p = oracle_mod.check_and_profile(claimed, ref, tau, eps_rel=0.0)
    # element 1: 0/0 -> NaN error but d = 0 <= 0 passes; 3,4,5: NaN difference -> violation
    assert p["violations"] == 3
    assert p["nan_count"] == 4
    assert p["hist"][2047] == 4
    assert p["hist"][2040] == 1            # element 2: 1/0 = +inf
    assert p["hist"][0] == 1               # element 0: e = 0
    assert p["max_rel"] == np.inf
    # NaN tau is a violation as well
    q = oracle_mod.check_and_profile(ref[:1], ref[:1], np.array([np.nan], f32))
    assert q["violations"] == 1


def test_nearest_rank_rule(oracle_mod):
    # n = 1000: ranks 500, 990, 999.  Values: 499 at 2^-20, 490 at 2^-15, 9 at 2^-10, 2 at 2^-5
    e = np.concatenate([np.full(499, 2.0 ** -20), np.full(490, 2.0 ** -15),
                        np.full(9, 2.0 ** -10), np.full(2, 2.0 ** -5)])
    _rng(1).shuffle(e)
    ref = np.ones(1000, f32)
    claimed = (1 + e).astype(f32)
    tau = np.ones(1000, f32)
    p = oracle_mod.check_and_profile(claimed, ref, tau, eps_rel=0.0)
    assert p["p50_bin"] == (127 - 15) << 3       # rank 500 is the first 2^-15
    assert p["p99_bin"] == (127 - 10) << 3       # rank 990 is the first 2^-10
    assert p["p999_bin"] == (127 - 5) << 3       # rank 999 is the first 2^-5
    assert p["p50"] == f32(2.0 ** -15 * 1.125)   # upper edge: next of 8 bins per octave
    assert p["p99"] == f32(2.0 ** -10 * 1.125)
    assert p["max_rel"] == f32(2.0 ** -5)
    # one fewer small value shifts rank 500 down a class boundary
    e2 = np.concatenate([np.full(500, 2.0 ** -20), np.full(500, 2.0 ** -15)])
    p2 = oracle_mod.check_and_profile((1 + e2).astype(f32), ref, tau, eps_rel=0.0)
    assert p2["p50_bin"] == (127 - 20) << 3
    # tiny n: rank = max(1, ceil(n p))
    for n, want in ((1, (0, 0, 0)), (3, (1, 2, 2))):
        vals = np.array([2.0 ** -20, 2.0 ** -15, 2.0 ** -10][:n])
        pp = oracle_mod.check_and_profile((1 + vals).astype(f32), np.ones(n, f32), np.ones(n, f32), eps_rel=0.0)
        bins = [(127 - 20) << 3, (127 - 15) << 3, (127 - 10) << 3]
        assert (pp["p50_bin"], pp["p99_bin"], pp["p999_bin"]) == tuple(bins[i] for i in want)
    empty = oracle_mod.check_and_profile(np.zeros(0, f32), np.zeros(0, f32), np.zeros(0, f32))
    assert empty["n"] == 0 and empty["accept"] == 1 and empty["hist"].sum() == 0


def test_histogram_percentiles_match_exact_order_statistics(oracle_mod):
    rng = _rng(33)
    n = 200003
    ref = rng.standard_normal(n).astype(f32)
    claimed = (ref.astype(np.float64) * (1 + rng.standard_normal(n) * 10.0 ** rng.uniform(-8, -3, n))).astype(f32)
    tau = (np.abs(ref) * 1e-5).astype(f32)
    p = oracle_mod.check_and_profile(claimed, ref, tau, eps_rel=1e-12)
    rd, cd = ref.astype(np.float64), claimed.astype(np.float64)
    e = (np.abs(cd - rd) / (np.abs(rd) + 1e-12)).astype(f32)       # IEEE binary64, then one cast
    assert np.array_equal(e, oracle_mod.rel_errors(claimed, ref, eps_rel=1e-12))
    es = np.sort(e)
    for name, num, den in (("p50", 1, 2), ("p99", 99, 100), ("p999", 999, 1000)):
        rank = max(1, -(-n * num // den))
        stat = es[rank - 1]
        assert _bin(stat) == p[name + "_bin"]
        assert stat < p[name] and p[name] <= stat * f32(1.126)
    assert p["max_rel"] == es[-1]
    assert p["violations"] == int(np.count_nonzero(~(np.abs(cd - rd) <= tau.astype(np.float64))))
    bins = (e.view(np.uint32) >> 20).astype(np.int64)
    assert np.array_equal(np.bincount(bins, minlength=2048), p["hist"])


def test_ulp_noise_profile_closed_form(oracle_mod):
    # claimed = ref moved by 0..3 ulps: relative error at most 3 * 2^-23 (eps = 0)
    rng = _rng(34)
    ref = rng.standard_normal(8192).astype(f32)
    k = rng.integers(0, 4, 8192) * rng.choice([-1, 1], 8192)
    claimed = (ref.view(np.int32) + k.astype(np.int32)).view(f32)
    tau = np.full(8192, 1e-3, f32)
    p = oracle_mod.check_and_profile(claimed, ref, tau, eps_rel=0.0)
    assert p["violations"] == 0 and p["accept"] == 1
    assert 0 < p["max_rel"] <= f32(3 * 2.0 ** -23)
    assert p["hist"][0] == int(np.count_nonzero(k == 0))
