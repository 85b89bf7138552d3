"""Pins for the oracle's error profiles on the paper's 22-point grid and the selection
statistic of Sec. 5.3 (errors of Sec. 3.2 Eq. 1-2): constructed cases with known ranks,
exact order statistics by sorting, hand-computed ratios."""
import numpy as np
import pytest

f32 = np.float32


def _bin(v):
    return int(np.array([v], f32).view(np.uint32)[0] >> 20)


def _edge(b):
    return np.array([(b + 1) << 20], np.uint32).view(f32)[0]


def test_grid_is_the_papers_22_points(oracle_mod):
    assert oracle_mod.GRID_PERCENT == [1, 5, 10, 15, 20, 25, 30, 35, 40, 45, 50, 55, 60, 65, 70, 75, 80,
                                       85, 90, 95, 99, 100]
    assert oracle_mod.NGRID == 22


def test_constructed_ranks(oracle_mod):
    # 100 elements with relative error j * 2^-20, j = 1..100 (eps = 0, ref = 1): the p-th
    # percentile by nearest rank is the p-th smallest, i.e. p * 2^-20
    j = np.arange(1, 101)
    ref = np.ones(100, f32)
    claimed = (1 + j * 2.0 ** -20).astype(f32)
    np.random.Generator(np.random.Philox(3)).shuffle(claimed)
    p = oracle_mod.profile_errors(claimed, ref, eps_rel=0.0)
    for g, pct in enumerate(oracle_mod.GRID_PERCENT):
        want = f32(pct * 2.0 ** -20)
        assert p["rel_bin"][g] == _bin(want) and p["abs_bin"][g] == _bin(want)
        assert p["rel_p"][g] == min(_edge(_bin(want)), f32(100 * 2.0 ** -20))
        assert want <= p["rel_p"][g] <= want * f32(1.126)
    assert p["rel_p"][-1] == p["max_rel"] == f32(100 * 2.0 ** -20)
    assert p["nan_count"] == 0 and np.isnan(p["p_max"]) and p["offending"] == 0


def test_abs_and_rel_are_different_things(oracle_mod):
    ref = np.array([4.0, -8.0], f32)
    claimed = np.array([5.0, -8.5], f32)
    p = oracle_mod.profile_errors(claimed, ref, eps_rel=0.0)
    assert p["max_abs"] == 1.0 and p["max_rel"] == 0.25
    assert p["hist_abs"][_bin(1.0)] == 1 and p["hist_abs"][_bin(0.5)] == 1
    assert p["hist_rel"][_bin(0.25)] == 1 and p["hist_rel"][_bin(0.0625)] == 1
    # eps enters the relative error only
    q = oracle_mod.profile_errors(claimed, ref, eps_rel=4.0)
    assert q["max_abs"] == 1.0 and q["max_rel"] == f32(1.0 / 8.0)


def test_against_sorting(oracle_mod):
    rng = np.random.Generator(np.random.Philox(44))
    n = 50021
    ref = rng.standard_normal(n).astype(f32)
    claimed = (ref.astype(np.float64) * (1 + rng.standard_normal(n) * 10.0 ** rng.uniform(-8, -2, n))).astype(f32)
    p = oracle_mod.profile_errors(claimed, ref, eps_rel=1e-12)
    d = np.abs(claimed.astype(np.float64) - ref.astype(np.float64))
    ea = np.sort(d.astype(f32))
    er = np.sort((d / (np.abs(ref.astype(np.float64)) + 1e-12)).astype(f32))
    for g, pct in enumerate(oracle_mod.GRID_PERCENT):
        rank = max(1, -(-n * pct // 100))
        for srt, bins, vals in ((ea, p["abs_bin"], p["abs_p"]), (er, p["rel_bin"], p["rel_p"])):
            stat = srt[rank - 1]
            assert _bin(stat) == bins[g]
            assert stat <= vals[g] <= max(stat * f32(1.126), _edge(0))
    assert p["max_abs"] == ea[-1] and p["max_rel"] == er[-1]
    assert np.array_equal(np.bincount(ea.view(np.uint32) >> 20, minlength=2048), p["hist_abs"])
    assert np.all(np.diff(p["abs_p"]) >= 0) and np.all(np.diff(p["rel_p"]) >= 0)


def test_selection_statistic(oracle_mod):
    rng = np.random.Generator(np.random.Philox(45))
    ref = rng.standard_normal(4096).astype(f32)
    claimed = (ref * (1 + 1e-5 * rng.standard_normal(4096))).astype(f32)
    base = oracle_mod.profile_errors(claimed, ref)
    # thresholds = alpha * profile with alpha = 3 (Sec. 3.2 threshold construction): ratio 1/3
    p = oracle_mod.profile_errors(claimed, ref, thr_abs=3 * base["abs_p"], thr_rel=3 * base["rel_p"])
    want = max(np.max(base["abs_p"].astype(np.float64) / (3 * base["abs_p"]).astype(f32)),
               np.max(base["rel_p"].astype(np.float64) / (3 * base["rel_p"]).astype(f32)))
    assert p["p_max"] == want and abs(p["p_max"] - 1 / 3) < 1e-7 and p["offending"] == 0
    # one threshold below the observed percentile: offending
    ta, tr = 3 * base["abs_p"], 3 * base["rel_p"]
    tr[10] = base["rel_p"][10] / f32(2)
    q = oracle_mod.profile_errors(claimed, ref, thr_abs=ta, thr_rel=tr)
    assert q["p_max"] == 2.0 and q["offending"] == 1
    # identical outputs: every error is 0, 0/0 ratios are skipped, 0/thr = 0
    z = oracle_mod.profile_errors(ref, ref, thr_abs=np.zeros(22, f32), thr_rel=np.ones(22, f32))
    assert z["p_max"] == 0.0 and z["offending"] == 0 and z["max_abs"] == 0.0


def test_nan_and_empty(oracle_mod):
    ref = np.array([1.0, np.nan, 2.0], f32)
    claimed = np.array([1.5, 1.0, np.inf], f32)
    p = oracle_mod.profile_errors(claimed, ref, eps_rel=0.0)
    assert p["nan_count"] == 1 and p["hist_rel"][2047] == 1 and p["hist_abs"][2047] == 1
    assert p["hist_abs"][2040] == 1 and p["max_abs"] == np.inf
    assert np.isnan(p["rel_p"][-1])           # the largest rank lands in the NaN bin
    e = oracle_mod.profile_errors(np.zeros(0, f32), np.zeros(0, f32))
    assert e["n"] == 0 and e["hist_abs"].sum() == 0


# ---------------------------------------------------------------- calibration (Sec. 3.2)

def test_envelope_is_the_pointwise_maximum(oracle_mod):
    rng = np.random.Generator(np.random.Philox(46))
    runs = [(rng.random(22).astype(f32), rng.random(22).astype(f32)) for _ in range(7)]
    ea, er, ta, tr = oracle_mod.calibrate_thresholds(runs, alpha=3.0)
    assert np.array_equal(ea, np.max([a for a, _ in runs], axis=0))
    assert np.array_equal(er, np.max([r for _, r in runs], axis=0))
    # thresholds: never below 3 x envelope, and within one binary32 step of it
    for env, thr in ((ea, ta), (er, tr)):
        exact = 3.0 * env.astype(np.float64)
        assert np.all(thr.astype(np.float64) >= exact)
        assert np.all(thr.astype(np.float64) <= exact * (1 + 2.0 ** -23))
    # order of the runs does not matter; one more run never lowers a threshold
    ea2, er2, ta2, tr2 = oracle_mod.calibrate_thresholds(runs[::-1], alpha=3.0)
    assert np.array_equal(ta, ta2) and np.array_equal(tr, tr2)
    more = runs + [(rng.random(22).astype(f32) * 2, rng.random(22).astype(f32) * 2)]
    _, _, ta3, tr3 = oracle_mod.calibrate_thresholds(more, alpha=3.0)
    assert np.all(ta3 >= ta) and np.all(tr3 >= tr) and np.any(ta3 > ta)


def test_threshold_values_by_hand(oracle_mod):
    a = np.full(22, 0.25, f32); r = np.full(22, 2.0 ** -20, f32)
    b = np.full(22, 0.125, f32); q = np.full(22, 2.0 ** -19, f32)
    ea, er, ta, tr = oracle_mod.calibrate_thresholds([(a, r), (b, q)], alpha=3.0)
    assert np.all(ea == 0.25) and np.all(er == f32(2.0 ** -19))
    assert np.all(ta == 0.75) and np.all(tr == f32(3 * 2.0 ** -19))        # exact products
    # a product that is not a binary32 number is rounded up: 3 x (1 + 2^-23) = 3 + 3 x 2^-23
    x = np.full(22, 1 + 2.0 ** -23, f32)
    _, _, t, _ = oracle_mod.calibrate_thresholds([(x, x)], alpha=3.0)
    assert np.all(t == f32(3 + 4 * 2.0 ** -23)) and np.all(t.astype(np.float64) > 3 * (1 + 2.0 ** -23))
    # NaN entries are skipped unless every run is NaN there; infinities propagate
    n1 = a.copy(); n1[3] = np.nan; n2 = b.copy(); n2[3] = np.nan; n2[5] = np.inf
    ea, _, ta, _ = oracle_mod.calibrate_thresholds([(n1, r), (n2, q)], alpha=2.0)
    assert np.isnan(ea[3]) and np.isnan(ta[3]) and ea[5] == np.inf and ta[5] == np.inf and ea[4] == 0.25
    n2[3] = 0.5
    ea, _, ta, _ = oracle_mod.calibrate_thresholds([(n1, r), (n2, q)], alpha=2.0)
    assert ea[3] == 0.5 and ta[3] == 1.0
    with pytest.raises(ValueError):
        oracle_mod.calibrate_thresholds([], alpha=3.0)


def test_calibrated_runs_are_never_offending(oracle_mod):
    """Thresholds built from a set of runs accept every one of those runs with p_max <= 1/alpha
    (the property the paper relies on: honest executions on calibrated hardware never trip the
    selection rule), and a run with 10x larger errors is offending."""
    rng = np.random.Generator(np.random.Philox(47))
    ref = rng.standard_normal(20000).astype(f32)
    runs = [(ref * (1 + s * rng.standard_normal(20000))).astype(f32) for s in (1e-6, 2e-6, 5e-7, 3e-6)]
    profs = [oracle_mod.profile_errors(c, ref) for c in runs]
    _, _, ta, tr = oracle_mod.calibrate_thresholds([(p["abs_p"], p["rel_p"]) for p in profs], alpha=3.0)
    for c in runs:
        p = oracle_mod.profile_errors(c, ref, thr_abs=ta, thr_rel=tr)
        assert p["offending"] == 0 and p["p_max"] <= 1 / 3 + 1e-7
    bad = (ref * (1 + 3e-5 * rng.standard_normal(20000))).astype(f32)
    assert oracle_mod.profile_errors(bad, ref, thr_abs=ta, thr_rel=tr)["offending"] == 1
