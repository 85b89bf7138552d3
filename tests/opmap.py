"""Run one traced operator (tao_inputs.Op) through the CPU oracle or the GPU library."""
import numpy as np

_NORM = {"layernorm": 0, "rmsnorm": 1, "bn_affine": 2, "sum": 3, "mean": 4}
_ACT = {"gelu": 0, "silu": 1, "mul": 2, "add": 3, "relu": 4}


def _np(t):
    return None if t is None else t.detach().cpu().numpy()


def oracle_tau(oracle, op, model=None):
    a = op.args
    if op.kind == "linear":
        return oracle.bound_linear(_np(a["A"]), _np(a["W"]), _np(a.get("bias")),
                                   trans_w=bool(op.attrs.get("trans_w", 0)), model=model)
    if op.kind == "softmax":
        return oracle.bound_softmax(_np(a["x"]), _np(op.y_ref), model=model)
    if op.kind in ("layernorm", "rmsnorm"):
        return oracle.bound_norm(_NORM[op.kind], _np(a["x"]), y=_np(op.y_ref), g=_np(a.get("gamma")),
                                 b=_np(a.get("beta")), eps=op.attrs["eps"], model=model)
    if op.kind == "bn_affine":
        return oracle.bound_norm(2, _np(a["x"]), y=_np(op.y_ref), g=_np(a["scale"]), b=_np(a["shift"]), model=model)
    if op.kind in ("sum", "mean"):
        return oracle.bound_norm(_NORM[op.kind], _np(a["x"]), y=_np(op.y_ref), model=model)
    if op.kind == "rope":
        return oracle.bound_rope(_np(a["x"]), _np(a["cos"]), _np(a["sin"]), inner=op.attrs["inner"], model=model)
    return oracle.bound_act(_ACT[op.kind], _np(a.get("x")), _np(op.y_ref), x2=_np(a.get("x2")), model=model)


def gpu_tau(tao, op, model=None, device="cuda"):
    def d(t):
        return None if t is None else t.to(device)
    a = op.args
    if op.kind == "linear":
        return tao.tao_bound_linear(d(a["A"]), d(a["W"]), d(a.get("bias")),
                                    trans_w=bool(op.attrs.get("trans_w", 0)), model=model)
    if op.kind == "softmax":
        return tao.tao_bound_softmax(d(a["x"]), d(op.y_ref), model=model)
    if op.kind in ("layernorm", "rmsnorm"):
        return tao.tao_bound_norm(_NORM[op.kind], d(a["x"]), d(op.y_ref), d(a.get("gamma")), d(a.get("beta")),
                                  eps=op.attrs["eps"], model=model)
    if op.kind == "bn_affine":
        return tao.tao_bound_norm(2, d(a["x"]), d(op.y_ref), d(a["scale"]), d(a["shift"]), model=model)
    if op.kind in ("sum", "mean"):
        return tao.tao_bound_norm(_NORM[op.kind], d(a["x"]), d(op.y_ref), model=model)
    if op.kind == "rope":
        return tao.tao_bound_rope(d(a["x"]), d(a["cos"]), d(a["sin"]), inner=op.attrs["inner"], model=model)
    return tao.tao_bound_act(_ACT[op.kind], d(a.get("x")), d(op.y_ref), x2=d(a.get("x2")), model=model)


REL_TOL = 1e-6      # spec tolerance: oracle <= gpu <= oracle * (1 + 1e-6)


def assert_bound_parity(tau_gpu, tau_or, what="", rel_tol=REL_TOL):
    """Element by element: NaN pattern identical, never below the oracle, within rel_tol above."""
    g = np.asarray(tau_gpu, dtype=np.float64).reshape(-1)
    o = np.asarray(tau_or, dtype=np.float64).reshape(-1)
    assert g.shape == o.shape, what
    nan_g, nan_o = np.isnan(g), np.isnan(o)
    assert np.array_equal(nan_g, nan_o), "%s: NaN pattern differs (%d vs %d)" % (what, nan_g.sum(), nan_o.sum())
    ok = ~nan_o
    g, o = g[ok], o[ok]
    below = g < o
    assert not below.any(), "%s: %d elements below the oracle, worst ratio %.3e" % (
        what, below.sum(), (g[below] / o[below]).min())
    above = g > o * (1.0 + rel_tol)
    assert not above.any(), "%s: %d elements above tolerance, worst excess %.3e" % (
        what, above.sum(), (g[above] / np.maximum(o[above], 1e-300) - 1).max())
    pos = o > 0
    return float((g[pos] / o[pos] - 1).max()) if pos.any() else 0.0


def assert_profile_equal(pg, po, what=""):
    for key in ("n", "violations", "nan_count", "accept", "p50_bin", "p99_bin", "p999_bin"):
        assert pg[key] == po[key], "%s: %s differs: gpu %r oracle %r" % (what, key, pg[key], po[key])
    assert np.array_equal(pg["hist"], po["hist"]), what + ": histogram differs"
    for key in ("max_rel", "p50", "p99", "p999"):
        a, b = np.float32(pg[key]), np.float32(po[key])
        assert (np.isnan(a) and np.isnan(b)) or a.view(np.uint32) == b.view(np.uint32), \
            "%s: %s differs: gpu %r oracle %r" % (what, key, a, b)
