"""GPU parity of the two projections of Sec. 4.4 against the CPU oracle: bit for bit (the caps
are binary64 formulas evaluated identically on both sides and equal magnitudes keep their index
order on both sides, so every output element is unique)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

f32 = np.float32
TILE = 4096


@pytest.fixture(scope="module")
def tao():
    import paper_2510_16028_amd as t
    t.lib()
    assert torch.cuda.is_available()
    return t


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _bits(a):
    return np.ascontiguousarray(a, dtype=f32).view(np.uint32)


def _thr(rng, scale, monotone=True):
    t = np.abs(rng.standard_normal(22)) * scale
    return (np.sort(t) if monotone else t).astype(f32)


def _same(got, want, what):
    g, w = _bits(got.cpu().numpy()), _bits(want)
    nan = np.isnan(want)
    bad = np.nonzero((g != w) & ~nan)[0]
    assert bad.size == 0, "%s: %d elements differ, first at %d: gpu %r oracle %r" % (
        what, bad.size, bad[0], got.flatten()[int(bad[0])].item(), want.flatten()[bad[0]])
    assert np.array_equal(np.isnan(got.cpu().numpy()), nan), what


def _delta(rng, n, kind):
    if kind == "errors":          # what an honest re-execution differs by: ~1e-6 of outputs of mixed size
        y = rng.standard_normal(n) * 10.0 ** rng.uniform(-2, 2, n)
        return (y * rng.standard_normal(n) * 6e-8).astype(f32)
    if kind == "wide":            # every byte of the key varies
        return (rng.standard_normal(n) * 10.0 ** rng.uniform(-30, 10, n)).astype(f32)
    if kind == "ties":            # few distinct magnitudes, many exact zeros
        v = rng.integers(-6, 7, n).astype(f32) * f32(2.5e-7)
        v[rng.random(n) < 0.3] = 0.0
        v[rng.random(n) < 0.1] = -0.0
        return v
    if kind == "equal":
        v = np.full(n, 3e-6, f32); v[::3] *= -1
        return v
    if kind == "special":
        v = (rng.standard_normal(n) * 1e-6).astype(f32)
        idx = rng.integers(0, n, max(1, n // 50))
        v[idx] = rng.choice(np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-45, -1e-45, 3e38], f32), idx.size)
        return v
    raise ValueError(kind)


def test_clip_matches_the_oracle(tao, oracle_mod):
    rng = _rng(1)
    for n, alpha, off in ((1, 1.0, 0), (5, 1.0, 0), (1023, 0.5, 0), (100003, 1.0, 0), (100003, 0.37, 1), (262144, 3.0, 0)):
        print("clip n", n, "alpha", alpha, "offset", off, flush=True)
        d = _delta(rng, n + off, "special")
        t = np.abs(rng.standard_normal(n + off) * 1e-6).astype(f32)
        t[rng.integers(0, n + off, 3)] = 0.0
        dg, tg = torch.from_numpy(d).cuda()[off:], torch.from_numpy(t).cuda()[off:]
        out = tao.tao_project_clip(dg, tg, alpha)
        torch.cuda.synchronize()
        _same(out, oracle_mod.project_clip(d[off:], t[off:], alpha), "clip n=%d" % n)
    # in place
    dg2 = dg.clone()
    tao.tao_project_clip(dg2, tg, alpha, out=dg2)
    _same(dg2, oracle_mod.project_clip(d[off:], t[off:], alpha), "clip in place")
    assert tao.tao_project_clip(torch.empty(0, device="cuda"), torch.empty(0, device="cuda")).numel() == 0


SIZES = [1, 2, 63, 64, 65, 1000, TILE - 1, TILE, TILE + 1, 8 * TILE + 37, 16 * TILE, 300001]


@pytest.mark.parametrize("kind", ["errors", "wide", "ties", "equal", "special"])
def test_empirical_projection_matches_the_oracle(tao, oracle_mod, kind):
    rng = _rng(hash(kind) % 1000 + 7)
    for n in SIZES:
        d = _delta(rng, n, kind)
        thr = _thr(rng, 2e-6 if kind != "wide" else 1e-3)
        alpha = float(rng.choice([1.0, 2.0, 3.0]))
        print("empirical", kind, "n", n, "alpha", alpha, flush=True)
        out = tao.tao_project_empirical(torch.from_numpy(d).cuda(), torch.from_numpy(thr).cuda(), alpha)
        torch.cuda.synchronize()
        want = oracle_mod.project_empirical(d, thr, alpha)
        _same(out, want, "%s n=%d" % (kind, n))
        clipped = int(np.sum(_bits(want) != _bits(d)))
        print("   clipped", clipped, "of", n, flush=True)


def test_empirical_projection_threshold_tables(tao, oracle_mod):
    rng = _rng(21)
    n = 5 * TILE + 11
    d = _delta(rng, n, "errors")
    dg = torch.from_numpy(d).cuda()
    tables = {"not monotone": _thr(rng, 2e-7, monotone=False), "zeros": np.zeros(22, f32),
              "huge": np.full(22, 3e38, f32), "steps": np.repeat(np.array([1e-8, 1e-7], f32), 11),
              "tiny": np.full(22, 1e-45, f32)}
    for name, thr in tables.items():
        for alpha in (1.0, 3.0, 0.0):
            print("table", name, "alpha", alpha, flush=True)
            out = tao.tao_project_empirical(dg, torch.from_numpy(thr).cuda(), alpha)
            torch.cuda.synchronize()
            _same(out, oracle_mod.project_empirical(d, thr, alpha), "%s alpha=%g" % (name, alpha))
    # in place, a caller's workspace, a multi-dimensional tensor, the empty tensor
    thr = tables["not monotone"]
    m = dg[: 4 * 32 * 160].reshape(4, 32, 160).clone()
    ws = torch.empty(tao.tao_project_workspace_bytes(m.numel()), dtype=torch.uint8, device="cuda")
    tao.tao_project_empirical(m, torch.from_numpy(thr).cuda(), 2.0, out=m, ws=ws)
    torch.cuda.synchronize()
    _same(m, oracle_mod.project_empirical(d[: m.numel()].reshape(4, 32, 160), thr, 2.0), "in place")
    assert tao.tao_project_empirical(torch.empty(0, device="cuda"), torch.from_numpy(thr).cuda()).numel() == 0
    with pytest.raises(tao.TaoError):
        tao.tao_project_empirical(dg, torch.from_numpy(thr).cuda(), 1.0, ws=ws[:4096])


def test_projection_with_calibrated_thresholds_end_to_end(tao, oracle_mod):
    """Thresholds as tao_calibrate_thresholds leaves them on the device; a perturbation ten times the
    honest error is projected back until the selection statistic of Sec. 5.3 no longer flags it."""
    rng = _rng(22)
    n = 70001
    ref = torch.from_numpy((rng.standard_normal(n) * 3).astype(f32))
    runs = [ref * (1 + 1e-6 * torch.from_numpy(rng.standard_normal(n).astype(f32))) for _ in range(3)]
    import ctypes
    bufs = torch.empty((3, ctypes.sizeof(tao.ErrorProfile)), dtype=torch.uint8, device="cuda")
    for i, c in enumerate(runs):
        tao.tao_profile_errors(c.cuda(), ref.cuda(), out=bufs[i], readback=False)
    ea, er, ta, tr = tao.tao_calibrate_thresholds(bufs, alpha=1.0)
    delta = (ref * 1e-5 * torch.from_numpy(rng.standard_normal(n).astype(f32)))
    for alpha in (1.0, 3.0):
        out = tao.tao_project_empirical(delta.cuda(), ta, alpha)
        torch.cuda.synchronize()
        _same(out, oracle_mod.project_empirical(delta.numpy(), ta.cpu().numpy(), alpha), "calibrated alpha=%g" % alpha)
        # order statistics whose rank lies at or below a grid point sit under alpha x its threshold
        srt = np.sort(np.abs(out.cpu().numpy()))
        caps = np.maximum.accumulate(ta.cpu().numpy().astype(np.float64)) * alpha
        for g, p in enumerate(oracle_mod.GRID_PERCENT):
            k = int(np.floor(n * p / 100.0 + 0.5))              # largest k with (k - 1/2)/n <= p/100
            assert k >= 1 and float(srt[k - 1]) <= caps[g], (g, p)
        assert np.any(out.cpu().numpy() != delta.numpy())


def test_library_calls_replay_from_a_hip_graph(tao, oracle_mod):
    """The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a sequence of them can be captured once and replayed.  Three replays on
    fresh inputs, with eager work and synchronisations in between, each compared bit for bit with
    the eager result of the same calls."""
    rng = _rng(31)
    M, N, K = 384, 256, 320
    A = torch.empty((M, K), device="cuda"); W = torch.empty((N, K), device="cuda")
    x = torch.empty((M, N), device="cuda")
    thr = torch.from_numpy(_thr(rng, 2e-6)).cuda()
    tau_f = torch.empty((M, N), device="cuda"); tau_s = torch.empty((M, N), device="cuda")
    tau_sm = torch.empty((M, N), device="cuda"); y_sm = torch.empty((M, N), device="cuda")
    proj = torch.empty((M, N), device="cuda"); claimed = torch.empty((M, N), device="cuda"); ref = torch.empty((M, N), device="cuda")
    prof = tao.new_profile_buffer(A.device)
    ws_split = torch.empty(tao.tao_linear_split_workspace_bytes(M, N, K, 1, True), dtype=torch.uint8, device="cuda")
    ws_proj = torch.empty(tao.tao_project_workspace_bytes(M * N), dtype=torch.uint8, device="cuda")
    ws_chk = torch.empty(tao.tao_check_workspace_bytes(M * N), dtype=torch.uint8, device="cuda")
    # the matmul bound checked in one call, both routes: in the epilogue (asked for by flag: K = 320 would
    # take the other route) and, on the first 96 columns of the same operands, through the stored bound
    # and the streaming check
    KS = 96
    prof_e = tao.new_profile_buffer(A.device); prof_s = tao.new_profile_buffer(A.device)
    ws_e = torch.empty(tao.tao_bound_check_linear_workspace_bytes(M, N, K, 1, True), dtype=torch.uint8, device="cuda")
    ws_s = torch.empty(tao.tao_bound_check_linear_workspace_bytes(M, N, KS, 1, True), dtype=torch.uint8, device="cuda")
    ref_s = torch.empty((M, N), device="cuda"); claimed_s = torch.empty((M, N), device="cuda")
    assert not tao.tao_bound_check_linear_in_epilogue(M, N, KS)
    epi = tao.FpModel(flags=tao.FLAG_CHECK_IN_EPILOGUE)

    def fill(seed):
        g = torch.Generator(device="cuda").manual_seed(seed)
        A.normal_(generator=g); W.normal_(generator=g); x.normal_(generator=g)
        ref.copy_(A @ W.t())
        claimed.copy_(ref * (1 + 3e-7 * torch.randn((M, N), device="cuda", generator=g)))
        y_sm.copy_(torch.softmax(x, -1))
        ref_s.copy_(A[:, :KS] @ W[:, :KS].t())
        claimed_s.copy_(ref_s * (1 + 3e-7 * torch.randn((M, N), device="cuda", generator=g)))

    def calls():
        tao.tao_bound_linear(A, W, out=tau_f)
        tao.tao_bound_linear_split(A, W, out=tau_s, ws=ws_split)
        tao.tao_bound_softmax(x, y_sm, out=tau_sm)
        tao.tao_check_and_profile(claimed, ref, tau_f, out=prof, readback=False, ws=ws_chk)
        tao.tao_project_empirical(x, thr, 2.0, out=proj, ws=ws_proj)
        tao.tao_bound_check_linear(A, W, None, ref, claimed, model=epi, out=prof_e, ws=ws_e, readback=False)
        tao.tao_bound_check_linear(A[:, :KS], W[:, :KS], None, ref_s, claimed_s, out=prof_s, ws=ws_s, readback=False)

    outs = (tau_f, tau_s, tau_sm, proj)
    fill(100)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        calls()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    torch.cuda.synchronize()
    for seed in (101, 102, 103):
        print("graph replay, seed", seed, flush=True)
        fill(seed)
        for o in outs:
            o.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        got_prof = tao.read_profile(prof)
        got_more = [tao.read_profile(b) for b in (prof_e, prof_s)]
        for b in (prof_e, prof_s):
            b.zero_()
        for o in outs:
            o.fill_(-2.0)
        calls()
        torch.cuda.synchronize()
        for g_, o in zip(got, outs):
            assert bool((g_.view(torch.int32) == o.view(torch.int32)).all())
        eager_prof = tao.read_profile(prof)
        assert got_prof["violations"] == eager_prof["violations"] and np.array_equal(got_prof["hist"], eager_prof["hist"])
        for g_, b in zip(got_more, (prof_e, prof_s)):
            e_ = tao.read_profile(b)
            assert g_["n"] == e_["n"] == M * N and g_["violations"] == e_["violations"] and g_["max_rel"] == e_["max_rel"]
            assert np.array_equal(g_["hist"], e_["hist"])
        want = oracle_mod.project_empirical(x.cpu().numpy(), thr.cpu().numpy(), 2.0)
        assert np.array_equal(got[3].cpu().numpy().view(np.uint32), want.view(np.uint32))
