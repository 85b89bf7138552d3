"""Seeded random shapes, kinds and claims through every one-pass entry point: the profile of
tao_bound_check_* must equal, field for field, that of the bound kernel followed by
tao_check_and_profile (and, for the matmul, the oracle's check of the stored bound); the
order-statistic projection must equal the oracle's bit for bit.  Claims carry planted violations,
NaN, infinities and a random share of values identical to the reference."""
import numpy as np
import pytest
import torch

import tao_inputs
from opmap import assert_profile_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tao():
    import paper_2510_16028_amd as t
    t.lib()
    assert torch.cuda.is_available()
    return t


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_one_pass_entry_points_on_random_cases(tao, oracle_mod, seed):
    oracle = oracle_mod
    rng = np.random.Generator(np.random.Philox(seed))
    g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))

    def noisy(ref, scale):
        c = ref * (1 + scale * torch.randn(ref.shape, generator=g))
        n = ref.numel()
        if n > 10:
            f = c.reshape(-1)
            idx = torch.randint(0, n, (max(1, n // 500),), generator=g)
            f[idx] = f[idx] * 1.5 + 0.3
            if rng.random() < 0.5: f[int(rng.integers(n))] = float("nan")
            if rng.random() < 0.3: f[int(rng.integers(n))] = float("inf")
            eq = torch.rand(ref.shape, generator=g) < rng.random()
            c = torch.where(eq, ref, c)
        return c.contiguous()
    for case in range(250):
        which = int(rng.integers(6))
        alpha = float(rng.choice([0.5, 1.0, 3.0])); eps = float(rng.choice([0.0, 1e-12, 1e-6]))
        if which == 0:      # linear
            M, N, K = int(rng.integers(1, 700)), int(rng.integers(1, 700)), int(rng.choice([0, 1, 31, 32, 33, 64, 200, 600, 1024, 1025, 1400, int(rng.integers(0, 1500))]))
            batch = int(rng.choice([1, 1, 2, 3])); tw = bool(rng.integers(2)); hb = bool(rng.integers(2)) and batch == 1
            A = torch.randn((batch, M, K), generator=g); W = torch.randn((batch, K, N) if tw else (batch, N, K), generator=g)
            if batch == 1: A, W = A[0], W[0]
            b = torch.randn((N,), generator=g) if hb else None
            Wnk = W.transpose(-1, -2) if tw else W
            ref = (A @ Wnk.transpose(-1, -2)) if K else torch.zeros(A.shape[:-1] + (N,))
            if hb: ref = ref + b
            ref = ref.contiguous(); c = noisy(ref, 3e-7)
            Ag, Wg, bg = A.cuda(), W.cuda(), None if b is None else b.cuda()
            tau = tao.tao_bound_linear_split(Ag, Wg, bg, trans_w=tw)
            route = tao.FpModel(flags=tao.FLAG_CHECK_IN_EPILOGUE) if rng.integers(2) else None      # both routes of the entry point
            fused = tao.tao_bound_check_linear(Ag, Wg, bg, ref.cuda(), c.cuda(), trans_w=tw, alpha=alpha, eps_rel=eps, model=route)
            two = tao.tao_check_and_profile(c.cuda(), ref.cuda(), tau, alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, two, "linear %s" % ((M, N, K, batch, tw, hb),))
            po = oracle.check_and_profile(c.numpy(), ref.numpy(), tau.cpu().numpy(), alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, po, "linear oracle %s" % ((M, N, K, batch, tw, hb),))
        elif which == 1:    # act
            kind = int(rng.choice([0, 1, 2, 3, 4, 6, 10, 17]))
            n = int(rng.choice([1, 7, 1000, 4097, 300001, int(rng.integers(1, 3000000))]))
            x = torch.randn((n,), generator=g) * 3; ref = torch.randn((n,), generator=g) * 10 ** float(rng.integers(-5, 5))
            c = noisy(ref, 2e-7)
            needs_x = kind in (0, 17)
            fused = tao.tao_bound_check_act(kind, x.cuda() if needs_x else None, ref.cuda(), c.cuda(), alpha=alpha, eps_rel=eps)
            tau = tao.tao_bound_act(kind, x.cuda() if needs_x else None, ref.cuda())
            two = tao.tao_check_and_profile(c.cuda(), ref.cuda(), tau, alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, two, "act %d n=%d" % (kind, n))
        elif which == 2:    # norm
            kind = int(rng.integers(2)); rows = int(rng.integers(1, 400)); cols = int(rng.choice([1, 3, 64, 255, 768, 1024, 1100, 2048, 4096, 5000, 9000]))
            x = torch.randn((rows, cols), generator=g) * 2 + 0.3; gam = 1 + 0.1 * torch.randn((cols,), generator=g); bet = torch.randn((cols,), generator=g)
            ref = tao_inputs.layernorm_f32(x, gam, bet, 1e-5) if kind == 0 else tao_inputs.rmsnorm_f32(x, gam, 1e-5)
            c = noisy(ref, 2e-7)
            fused = tao.tao_bound_check_norm(kind, x.cuda(), ref.cuda(), c.cuda(), gam.cuda(), bet.cuda(), eps=1e-5, alpha=alpha, eps_rel=eps)
            tau = tao.tao_bound_norm(kind, x.cuda(), ref.cuda(), gam.cuda(), bet.cuda(), eps=1e-5)
            two = tao.tao_check_and_profile(c.cuda(), ref.cuda(), tau, alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, two, "norm %d %dx%d" % (kind, rows, cols))
        elif which == 3:    # softmax
            rows = int(rng.integers(1, 300)); cols = int(rng.choice([1, 5, 128, 500, 1024, 2048, 3000, 4096, 9000]))
            x = torch.randn((rows, cols), generator=g) * 3
            if cols > 4: x[rows // 2, cols // 2:] = float("-inf")
            ref = tao_inputs.softmax_f32(x); c = noisy(ref, 2e-7)
            fused = tao.tao_bound_check_softmax(x.cuda(), ref.cuda(), c.cuda(), alpha=alpha, eps_rel=eps)
            tau = tao.tao_bound_softmax(x.cuda(), ref.cuda())
            two = tao.tao_check_and_profile(c.cuda(), ref.cuda(), tau, alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, two, "softmax %dx%d" % (rows, cols))
        elif which == 4:    # rope
            d = int(rng.choice([2, 6, 8, 64, 128, 20])); inner = int(rng.choice([1, 2, 8])); npos = int(rng.integers(1, 40)); rows = inner * npos * int(rng.integers(1, 4))
            il = bool(rng.integers(2))
            x = torch.randn((rows, d), generator=g); ang = torch.rand((npos, d // 2), generator=g) * 6
            cs, sn = torch.cos(ang), torch.sin(ang)
            ref = torch.randn((rows, d), generator=g); c = noisy(ref, 2e-7)
            fused = tao.tao_bound_check_rope(x.cuda(), cs.cuda(), sn.cuda(), ref.cuda(), c.cuda(), inner=inner, interleaved=il, alpha=alpha, eps_rel=eps)
            tau = tao.tao_bound_rope(x.cuda(), cs.cuda(), sn.cuda(), inner=inner, interleaved=il)
            two = tao.tao_check_and_profile(c.cuda(), ref.cuda(), tau, alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, two, "rope %s" % ((rows, d, inner, npos, il),))
        else:               # projection
            n = int(rng.choice([1, 2, 100, 4096, 4097, 70000, int(rng.integers(1, 2000000))]))
            scale = 10.0 ** float(rng.integers(-8, 3))
            d = (torch.randn((n,), generator=g) * scale * torch.pow(10.0, torch.rand((n,), generator=g) * float(rng.integers(0, 6)))).numpy().astype(np.float32)
            if rng.random() < 0.5: d = np.round(d / (scale * 0.25)).astype(np.float32) * np.float32(scale * 0.25)   # ties
            thr = (np.abs(rng.standard_normal(22)) * scale * float(rng.choice([0.1, 1, 10]))).astype(np.float32)
            if rng.random() < 0.7: thr = np.sort(thr)
            out = tao.tao_project_empirical(torch.from_numpy(d).cuda(), torch.from_numpy(thr).cuda(), alpha).cpu().numpy()
            want = oracle.project_empirical(d, thr, alpha)
            assert np.array_equal(out.view(np.uint32), want.view(np.uint32)), ("projection", n, scale)
