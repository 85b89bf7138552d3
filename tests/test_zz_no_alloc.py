"""The entry point that allocates nothing (tao_check_and_profile_static: its partial histograms and
counters live in a fixed array inside the library) against tao_check_and_profile with a caller's
workspace: the same profile, field for field, on two calls in a row, the second on a smaller
input; and against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

from opmap import assert_profile_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tao():
    import paper_2510_16028_amd as t
    t.lib()
    assert torch.cuda.is_available()
    return t


def _case(seed, n):
    g = torch.Generator().manual_seed(seed)
    ref = torch.randn((n,), generator=g)
    tau = (ref.abs() * 2.0 ** -20 + 1e-9).contiguous()
    f = torch.rand((n,), generator=g) * 1.3                      # some claims beyond the bound
    sign = torch.where(torch.rand((n,), generator=g) < 0.5, -1.0, 1.0)
    claimed = (ref + sign * f * tau).contiguous()
    if n > 10:
        claimed[3] = float("nan"); tau[7] = float("nan"); claimed[9] = ref[9]
    return claimed, ref, tau


def test_static_entry_matches_the_workspace_entry_twice(tao, oracle_mod):
    # the output buffers exist before the calls: the entry point itself allocates nothing
    outs = [tao.new_profile_buffer(torch.device("cuda")) for _ in range(2)]
    results = []
    cases = [_case(1, 3_000_017), _case(2, 70_001)]              # the second call on a smaller input
    dev = [tuple(t.cuda() for t in c) for c in cases]
    torch.cuda.synchronize()
    for (c, r, t), out in zip(dev, outs):
        results.append(tao.tao_check_and_profile_static(c, r, t, alpha=1.0, eps_rel=1e-12, out=out, readback=False))
    torch.cuda.synchronize()
    for (c, r, t), (ch, rh, th), buf in zip(dev, cases, results):
        got = tao.read_profile(buf)
        want = tao.tao_check_and_profile(c, r, t, alpha=1.0, eps_rel=1e-12)
        assert_profile_equal(got, want, "static vs workspace, n = %d" % c.numel())
        assert_profile_equal(got, oracle_mod.check_and_profile(ch.numpy(), rh.numpy(), th.numpy(), alpha=1.0, eps_rel=1e-12),
                             "static vs oracle, n = %d" % c.numel())
        assert got["n"] == c.numel() and got["violations"] > 0 and got["nan_count"] >= 1


def test_static_entry_small_and_empty_inputs_after_a_large_one(tao, oracle_mod):
    big = _case(3, 1_500_000)
    tao.tao_check_and_profile_static(*(t.cuda() for t in big))
    for n in (0, 1, 5, 4097):
        c, r, t = _case(10 + n, n)
        got = tao.tao_check_and_profile_static(c.cuda(), r.cuda(), t.cuda(), alpha=2.0, eps_rel=1e-6)
        assert_profile_equal(got, oracle_mod.check_and_profile(c.numpy(), r.numpy(), t.numpy(), alpha=2.0, eps_rel=1e-6),
                             "static, n = %d" % n)


def test_static_entry_rejects_sizes_beyond_its_maximum(tao):
    c, r, t = (x.cuda() for x in _case(4, 64))
    out = tao.new_profile_buffer(c.device)
    L = tao.lib()
    vp = ctypes.c_void_p
    too_many = tao.STATIC_CHECK_MAX_N + 1
    rc = L.tao_check_and_profile_static(vp(c.data_ptr()), vp(r.data_ptr()), vp(t.data_ptr()), too_many,
                                        1.0, 1e-12, vp(out.data_ptr()), None)
    assert rc == tao.ERR_SHAPE                                   # nothing was enqueued
    rc = L.tao_check_and_profile_static(vp(c.data_ptr()), vp(r.data_ptr()), vp(t.data_ptr()), 64, 1.0, 1e-12, None, None)
    assert rc == tao.ERR_NULL
    torch.cuda.synchronize()
