"""CPU oracle for the TAO per-operator tolerance engine -- TEST INFRASTRUCTURE.

Thin ctypes/numpy front end of oracle/tao_oracle.c (plain C, binary64 with
directed rounding).  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path never does, and
this package imports nothing from the GPU library.
"""
import ctypes
import os

import numpy as np

from . import build as _build
from .project import cap_curve, project_clip, project_empirical  # noqa: F401  (Sec. 4.4)

NBINS = 2048

LAYERNORM, RMSNORM, BN_AFFINE, SUM, MEAN = 0, 1, 2, 3, 4
GELU_ERF, SILU, MUL, ADD, RELU = 0, 1, 2, 3, 4
SUB, DIV, EXACT, SQRT, RSQRT, EXP, LOG, SIN, COS, TANH, POW, SIGMOID, GELU_TANH = range(5, 18)
UNDERFLOW_TERMS = 1


class Model(ctypes.Structure):
    """Floating-point model (App. A.1) and intrinsic accuracy constants (Sec. 3.1)."""
    _fields_ = [("u", ctypes.c_double), ("mode", ctypes.c_int), ("lam", ctypes.c_double),
                ("c_exp", ctypes.c_double), ("c_erf", ctypes.c_double),
                ("c_rsqrt", ctypes.c_double), ("c_div", ctypes.c_double),
                ("flags", ctypes.c_uint),
                ("c_log", ctypes.c_double), ("c_sin", ctypes.c_double), ("c_cos", ctypes.c_double),
                ("c_tanh", ctypes.c_double), ("c_pow", ctypes.c_double)]

    def __init__(self, u=2.0 ** -24, mode=0, lam=4.0, c_exp=2.0, c_erf=2.0, c_rsqrt=2.0,
                 c_div=2.0, flags=0, c_log=2.0, c_sin=4.0, c_cos=4.0, c_tanh=4.0, c_pow=8.0):
        super().__init__(u, mode, lam, c_exp, c_erf, c_rsqrt, c_div, flags,
                         c_log, c_sin, c_cos, c_tanh, c_pow)


class Profile(ctypes.Structure):
    _fields_ = [("n", ctypes.c_uint64), ("violations", ctypes.c_uint64),
                ("nan_count", ctypes.c_uint64), ("max_rel", ctypes.c_float),
                ("accept", ctypes.c_uint32), ("p50_bin", ctypes.c_uint32),
                ("p99_bin", ctypes.c_uint32), ("p999_bin", ctypes.c_uint32),
                ("p50", ctypes.c_float), ("p99", ctypes.c_float), ("p999", ctypes.c_float),
                ("pad_", ctypes.c_uint32), ("hist", ctypes.c_uint64 * NBINS)]

    def as_dict(self):
        return {"n": int(self.n), "violations": int(self.violations),
                "nan_count": int(self.nan_count), "max_rel": float(self.max_rel),
                "accept": int(self.accept), "p50_bin": int(self.p50_bin),
                "p99_bin": int(self.p99_bin), "p999_bin": int(self.p999_bin),
                "p50": float(self.p50), "p99": float(self.p99), "p999": float(self.p999),
                "hist": np.ctypeslib.as_array(self.hist).copy()}


NGRID = 22
GRID_PERCENT = [1] + [5 * g for g in range(1, 20)] + [99, 100]


class ErrorProfile(ctypes.Structure):
    _fields_ = [("n", ctypes.c_uint64), ("nan_count", ctypes.c_uint64),
                ("max_abs", ctypes.c_float), ("max_rel", ctypes.c_float),
                ("abs_p", ctypes.c_float * NGRID), ("rel_p", ctypes.c_float * NGRID),
                ("abs_bin", ctypes.c_uint32 * NGRID), ("rel_bin", ctypes.c_uint32 * NGRID),
                ("p_max", ctypes.c_double), ("offending", ctypes.c_uint32), ("pad_", ctypes.c_uint32),
                ("hist_abs", ctypes.c_uint64 * NBINS), ("hist_rel", ctypes.c_uint64 * NBINS)]

    def as_dict(self):
        arr = lambda a: np.ctypeslib.as_array(a).copy()
        return {"n": int(self.n), "nan_count": int(self.nan_count), "max_abs": float(self.max_abs),
                "max_rel": float(self.max_rel), "abs_p": arr(self.abs_p), "rel_p": arr(self.rel_p),
                "abs_bin": arr(self.abs_bin), "rel_bin": arr(self.rel_bin), "p_max": float(self.p_max),
                "offending": int(self.offending), "hist_abs": arr(self.hist_abs), "hist_rel": arr(self.hist_rel)}


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        fp = ctypes.POINTER(ctypes.c_float)
        mp = ctypes.POINTER(Model)
        L.taoo_gamma.restype = ctypes.c_double
        L.taoo_gamma.argtypes = [ctypes.c_long, mp]
        L.taoo_bound_linear.argtypes = [fp, fp, fp, fp] + [ctypes.c_long] * 6 + [ctypes.c_int] + \
            [ctypes.c_long] * 4 + [mp]
        L.taoo_bound_softmax.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_long, ctypes.c_long, mp]
        L.taoo_bound_conv2d.argtypes = [fp, fp, fp, fp] + [ctypes.c_long] * 13 + [mp]
        L.taoo_bound_norm.argtypes = [ctypes.c_int, fp, fp, fp, fp, ctypes.c_double, fp,
                                      ctypes.c_long, ctypes.c_long, ctypes.c_long, mp]
        L.taoo_bound_act.argtypes = [ctypes.c_int, fp, fp, fp, fp, ctypes.c_long, mp]
        L.taoo_bound_rope.argtypes = [fp, fp, fp, fp] + [ctypes.c_long] * 4 + [ctypes.c_int, mp]
        L.taoo_check_and_profile.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_double,
                                             ctypes.c_double, ctypes.POINTER(Profile)]
        L.taoo_rel_errors.argtypes = [fp, fp, ctypes.c_long, ctypes.c_double, fp]
        L.taoo_profile_errors.argtypes = [fp, fp, ctypes.c_long, ctypes.c_double, fp, fp,
                                          ctypes.POINTER(ErrorProfile)]
        L.taoo_error_profile_size.restype = ctypes.c_size_t
        assert L.taoo_error_profile_size() == ctypes.sizeof(ErrorProfile)
        L.taoo_calibrate_thresholds.argtypes = [ctypes.POINTER(ErrorProfile), ctypes.c_long, ctypes.c_double,
                                                fp, fp, fp, fp]
        L.taoo_num_threads.restype = ctypes.c_int
        L.taoo_profile_size.restype = ctypes.c_size_t
        assert L.taoo_profile_size() == ctypes.sizeof(Profile)
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _chk(rc):
    if rc != 0:
        raise ValueError("oracle status %d" % rc)


def gamma(k, model=None):
    """Gamma(k) rounded up in binary64 (App. A.1 Eq. gamma-def; Sec. 3.1 probabilistic form)."""
    model = model or Model()
    return lib().taoo_gamma(int(k), ctypes.byref(model))


def bound_linear(A, W, bias=None, trans_w=False, model=None):
    """tau[..., M, N] for A[..., M, K] and W[..., N, K] (or [..., K, N] with trans_w)."""
    model = model or Model()
    A = _f32(A); W = _f32(W)
    batched = A.ndim == 3
    A3 = A if batched else A[None]
    W3 = W if W.ndim == 3 else W[None]
    B, M, K = A3.shape
    N = W3.shape[2] if trans_w else W3.shape[1]
    assert (W3.shape[1] if trans_w else W3.shape[2]) == K
    assert W3.shape[0] in (1, B)
    bias = None if bias is None else _f32(bias)
    tau = np.empty((B, M, N), dtype=np.float32)
    sW = 0 if W3.shape[0] == 1 else W3.shape[1] * W3.shape[2]
    _chk(lib().taoo_bound_linear(_p(A3), _p(W3), _p(bias), _p(tau), M, N, K, K, W3.shape[2], N,
                                 int(bool(trans_w)), B, M * K, sW, M * N, ctypes.byref(model)))
    return tau if batched else tau[0]


def conv_out_size(size, k, stride, pad, dil):
    return (size + 2 * pad - dil * (k - 1) - 1) // stride + 1


def bound_conv2d(x, w, bias=None, stride=(1, 1), padding=(0, 0), dilation=(1, 1), model=None):
    """tau[Nb, OH, OW, Cout] for x[Nb, H, W, C] (channels last) and w[Cout, R, S, C]."""
    model = model or Model()
    x = _f32(x); w = _f32(w)
    Nb, H, W, C = x.shape
    Cout, R, S, C2 = w.shape
    assert C == C2
    bias = None if bias is None else _f32(bias)
    if min(stride) < 1 or min(dilation) < 1 or min(padding) < 0:
        raise ValueError("bad convolution geometry")
    if min(H + 2 * padding[0] - dilation[0] * (R - 1), W + 2 * padding[1] - dilation[1] * (S - 1)) < 1:
        raise ValueError("filter larger than the padded input")
    OH = conv_out_size(H, R, stride[0], padding[0], dilation[0])
    OW = conv_out_size(W, S, stride[1], padding[1], dilation[1])
    tau = np.empty((Nb, OH, OW, Cout), dtype=np.float32)
    _chk(lib().taoo_bound_conv2d(_p(x), _p(w), _p(bias), _p(tau), Nb, H, W, C, Cout, R, S,
                                 stride[0], stride[1], padding[0], padding[1], dilation[0], dilation[1],
                                 ctypes.byref(model)))
    return tau


def bound_softmax(x, y, model=None):
    model = model or Model()
    x = _f32(x); y = _f32(y)
    cols = x.shape[-1]; rows = x.size // cols
    tau = np.empty_like(x)
    _chk(lib().taoo_bound_softmax(_p(x), _p(y), _p(tau), rows, cols, cols, ctypes.byref(model)))
    return tau


def bound_norm(kind, x, y=None, g=None, b=None, eps=0.0, model=None):
    model = model or Model()
    x = _f32(x)
    cols = x.shape[-1]; rows = x.size // cols
    y = None if y is None else _f32(y)
    g = None if g is None else _f32(g)
    b = None if b is None else _f32(b)
    if kind in (SUM, MEAN):
        tau = np.empty(x.shape[:-1], dtype=np.float32)
    else:
        tau = np.empty_like(x)
    _chk(lib().taoo_bound_norm(kind, _p(x), _p(y), _p(g), _p(b), float(eps), _p(tau), rows, cols,
                               cols, ctypes.byref(model)))
    return tau


def bound_groupnorm(x, y, groups, g=None, b=None, eps=0.0, model=None):
    """GroupNorm of x[N, C, *spatial] (channel-major, contiguous) with `groups` groups: each
    (sample, group) is a LayerNorm over its C/groups channels times all spatial positions, with
    the affine parameters of a channel repeated over that channel's positions.  Written as that
    definition: one LayerNorm bound per group on the rows gathered over the batch."""
    x = _f32(x); y = _f32(y)
    N, C = x.shape[0], x.shape[1]
    hw = int(np.prod(x.shape[2:], dtype=np.int64))
    if groups < 1 or C % groups:
        raise ValueError("channels must be a multiple of groups")
    cpg = C // groups
    xr = x.reshape(N, groups, cpg * hw); yr = y.reshape(N, groups, cpg * hw)
    tau = np.empty_like(xr)
    for j in range(groups):
        gj = None if g is None else np.repeat(_f32(g)[j * cpg:(j + 1) * cpg], hw)
        bj = None if b is None else np.repeat(_f32(b)[j * cpg:(j + 1) * cpg], hw)
        tau[:, j, :] = bound_norm(LAYERNORM, xr[:, j, :], y=yr[:, j, :], g=gj, b=bj, eps=eps, model=model)
    return tau.reshape(x.shape)


def bound_act(kind, x, y, x2=None, model=None):
    model = model or Model()
    y = _f32(y)
    x = None if x is None else _f32(x)
    x2 = None if x2 is None else _f32(x2)
    tau = np.empty_like(y)
    _chk(lib().taoo_bound_act(kind, _p(x), _p(x2), _p(y), _p(tau), y.size, ctypes.byref(model)))
    return tau


def bound_rope(x, cos, sin, inner=1, interleaved=False, model=None):
    """tau like x[..., d] for the rotation by the tables cos, sin [npos, d/2]; row r of the
    flattened x uses table row (r // inner) % npos."""
    model = model or Model()
    x = _f32(x); cos = _f32(cos); sin = _f32(sin)
    d = x.shape[-1]; rows = x.size // max(d, 1)
    if not (cos.shape == sin.shape and cos.ndim == 2 and cos.shape[1] * 2 == d):
        raise ValueError("cos and sin must be [npos, d/2] with d even")
    tau = np.empty_like(x)
    _chk(lib().taoo_bound_rope(_p(x), _p(cos), _p(sin), _p(tau), rows, d, int(inner), cos.shape[0],
                               int(bool(interleaved)), ctypes.byref(model)))
    return tau


def check_and_profile(claimed, ref, tau, alpha=1.0, eps_rel=1e-12):
    claimed = _f32(claimed); ref = _f32(ref); tau = _f32(tau)
    assert claimed.size == ref.size == tau.size
    out = Profile()
    _chk(lib().taoo_check_and_profile(_p(claimed), _p(ref), _p(tau), claimed.size, float(alpha),
                                      float(eps_rel), ctypes.byref(out)))
    return out.as_dict()


def rel_errors(claimed, ref, eps_rel=1e-12):
    claimed = _f32(claimed); ref = _f32(ref)
    out = np.empty(claimed.shape, dtype=np.float32)
    _chk(lib().taoo_rel_errors(_p(claimed), _p(ref), claimed.size, float(eps_rel), _p(out)))
    return out


def profile_errors(claimed, ref, eps_rel=1e-12, thr_abs=None, thr_rel=None):
    """Absolute / relative error profiles on the 22-point grid and the selection statistic (Sec. 5.3)."""
    claimed = _f32(claimed); ref = _f32(ref)
    assert claimed.size == ref.size
    ta = None if thr_abs is None else _f32(thr_abs)
    tr = None if thr_rel is None else _f32(thr_rel)
    assert (ta is None) == (tr is None)
    if ta is not None:
        assert ta.size == NGRID and tr.size == NGRID
    out = ErrorProfile()
    _chk(lib().taoo_profile_errors(_p(claimed), _p(ref), claimed.size, float(eps_rel), _p(ta), _p(tr),
                                   ctypes.byref(out)))
    return out.as_dict()


def calibrate_thresholds(profiles, alpha=3.0):
    """Max-envelope of the 22-point profiles of several runs and the alpha-scaled thresholds
    (Sec. 3.2).  profiles: list of (abs_p, rel_p) pairs of 22 float32 values each.
    Returns (env_abs, env_rel, thr_abs, thr_rel)."""
    arr = (ErrorProfile * len(profiles))()
    for i, (a, r) in enumerate(profiles):
        a = _f32(a); r = _f32(r)
        assert a.size == NGRID and r.size == NGRID
        for g in range(NGRID):
            arr[i].abs_p[g] = float(a[g]) if a[g] == a[g] else float("nan")
            arr[i].rel_p[g] = float(r[g]) if r[g] == r[g] else float("nan")
    out = [np.empty(NGRID, np.float32) for _ in range(4)]
    _chk(lib().taoo_calibrate_thresholds(arr, len(profiles), float(alpha), *[_p(o) for o in out]))
    return tuple(out)


def num_threads():
    return lib().taoo_num_threads()
