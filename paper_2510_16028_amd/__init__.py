"""Python binding of libtao.so, the MI355X per-operator tolerance engine.

Argument marshalling only: every function below hands device pointers, sizes
and the current HIP stream to the C entry point of the same name (declared in
include/tao.h); all arithmetic runs in the library's kernels.  PyTorch is used
for device memory and streams.  There is no CPU fallback: if the shared
library is missing or no GPU is present, calls raise.
"""
import ctypes
import os

import numpy as np

NBINS = 2048
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtao.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_K_RANGE, ERR_MODEL, ERR_KIND, ERR_LAUNCH, ERR_WORKSPACE = \
    -1, -2, -3, -4, -5, -6, -7, -8
MODE_DETERMINISTIC, MODE_PROBABILISTIC = 0, 1
FLAG_UNDERFLOW_TERMS, FLAG_FAST_ACCUM, FLAG_CHECK_IN_EPILOGUE = 1, 2, 4
NORM_LAYERNORM, NORM_RMSNORM, NORM_BN_AFFINE, NORM_SUM, NORM_MEAN = 0, 1, 2, 3, 4
ACT_GELU_ERF, ACT_SILU, ACT_MUL, ACT_ADD, ACT_RELU = 0, 1, 2, 3, 4
(ACT_SUB, ACT_DIV, ACT_EXACT, ACT_SQRT, ACT_RSQRT, ACT_EXP, ACT_LOG, ACT_SIN, ACT_COS, ACT_TANH,
 ACT_POW, ACT_SIGMOID, ACT_GELU_TANH) = range(5, 18)


class FpModel(ctypes.Structure):
    """tao_fp_model: unit roundoff, deterministic/probabilistic constant, intrinsic accuracies."""
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
    """tao_profile as laid out in device memory."""
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
    """tao_error_profile as laid out in device memory."""
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
                "offending": int(self.offending), "hist_abs": arr(self.hist_abs),
                "hist_rel": arr(self.hist_rel)}


class TaoError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().tao_status_string(status).decode()
        extra = ""
        if status == ERR_LAUNCH:
            extra = " (hipError %d)" % lib().tao_last_hip_error()
        super().__init__("%s: %s%s" % (where, msg, extra))


EXPORTS = ["tao_default_model", "tao_gamma", "tao_bound_linear", "tao_bound_linear_split",
           "tao_linear_split_workspace_bytes", "tao_linear_split_preferred",
           "tao_split_image_bytes", "tao_split_operand", "tao_bound_linear_images", "tao_linear_images_workspace_bytes",
           "tao_bound_check_linear_images", "tao_check_linear_images_workspace_bytes", "tao_bound_check_linear_in_epilogue",
           "tao_bound_check_linear", "tao_bound_check_linear_workspace_bytes", "tao_selftest_matrix_core_bf16", "tao_selftest_workspace_bytes", "tao_bound_conv2d",
           "tao_conv2d_split_supported", "tao_conv2d_split_workspace_bytes", "tao_bound_conv2d_split", "tao_bound_check_conv2d", "tao_bound_softmax",
           "tao_bound_norm", "tao_bound_groupnorm", "tao_groupnorm_workspace_bytes", "tao_bound_act", "tao_bound_check_act", "tao_bound_rope", "tao_bound_check_rope", "tao_bound_check_norm", "tao_check_and_profile",
           "tao_check_and_profile_static",
           "tao_check_workspace_bytes", "tao_bound_check_softmax", "tao_profile_errors", "tao_profile_workspace_bytes",
           "tao_calibrate_thresholds", "tao_project_clip", "tao_project_empirical", "tao_project_workspace_bytes",
           "tao_selftest_matrix_core", "tao_last_hip_error", "tao_status_string"]

_lib = None


def lib():
    """Load libtao.so (built by `python -m paper_2510_16028_amd.build`); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libtao.so not built: run `python -m paper_2510_16028_amd.build` "
                           "(there is no CPU fallback)")
    # torch brings its own copy of the HIP runtime; load it first so that libtao.so binds to the
    # same one (two runtimes in one process do not share a device context)
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, lg, dbl = ctypes.c_void_p, ctypes.c_long, ctypes.c_double
    mp = ctypes.POINTER(FpModel)
    L.tao_default_model.argtypes = [mp]
    L.tao_default_model.restype = None
    L.tao_gamma.argtypes = [lg, mp]
    L.tao_gamma.restype = dbl
    L.tao_bound_linear.argtypes = [vp, vp, vp, vp, lg, lg, lg, lg, lg, lg, ctypes.c_int,
                                   lg, lg, lg, lg, mp, vp]
    L.tao_bound_linear_split.argtypes = [vp, vp, vp, vp, lg, lg, lg, lg, lg, lg, ctypes.c_int,
                                         lg, lg, lg, lg, mp, vp, ctypes.c_size_t, vp]
    L.tao_bound_check_linear.argtypes = [vp, vp, vp, vp, vp, vp, lg, lg, lg, lg, lg, lg, ctypes.c_int,
                                         lg, lg, lg, lg, dbl, dbl, mp, vp, vp, ctypes.c_size_t, vp]
    L.tao_bound_check_linear_workspace_bytes.argtypes = [lg, lg, lg, lg, ctypes.c_int]
    L.tao_bound_check_linear_workspace_bytes.restype = ctypes.c_size_t
    L.tao_linear_split_workspace_bytes.argtypes = [lg, lg, lg, lg, ctypes.c_int]
    L.tao_linear_split_workspace_bytes.restype = ctypes.c_size_t
    L.tao_linear_split_preferred.argtypes = [lg, lg, lg, lg]
    L.tao_split_image_bytes.argtypes = [lg, lg, lg]
    L.tao_split_image_bytes.restype = ctypes.c_size_t
    L.tao_split_operand.argtypes = [vp, lg, lg, lg, ctypes.c_int, lg, lg, vp, ctypes.c_size_t, vp]
    L.tao_bound_linear_images.argtypes = [vp, vp, vp, vp, lg, lg, lg, lg, lg, lg, ctypes.c_int, mp, vp, ctypes.c_size_t, vp]
    L.tao_linear_images_workspace_bytes.argtypes = [lg, lg, lg, lg]
    L.tao_linear_images_workspace_bytes.restype = ctypes.c_size_t
    L.tao_bound_check_linear_images.argtypes = [vp, vp, vp, vp, vp, vp, lg, lg, lg, lg, lg, lg, ctypes.c_int, dbl, dbl, mp, vp,
                                                vp, ctypes.c_size_t, vp]
    L.tao_check_linear_images_workspace_bytes.argtypes = [lg, lg, lg, lg]
    L.tao_check_linear_images_workspace_bytes.restype = ctypes.c_size_t
    L.tao_bound_check_linear_in_epilogue.argtypes = [lg, lg, lg, lg]
    L.tao_selftest_matrix_core_bf16.argtypes = [ctypes.POINTER(ctypes.c_uint), lg, vp, ctypes.c_size_t, vp]
    L.tao_selftest_workspace_bytes.argtypes = [lg]
    L.tao_selftest_workspace_bytes.restype = ctypes.c_size_t
    L.tao_bound_conv2d.argtypes = [vp, vp, vp, vp] + [lg] * 13 + [mp, vp]
    L.tao_conv2d_split_supported.argtypes = [lg] * 13
    L.tao_conv2d_split_workspace_bytes.argtypes = [lg] * 13 + [ctypes.c_int]
    L.tao_conv2d_split_workspace_bytes.restype = ctypes.c_size_t
    L.tao_bound_conv2d_split.argtypes = [vp, vp, vp, vp] + [lg] * 13 + [mp, vp, ctypes.c_size_t, vp]
    L.tao_bound_check_conv2d.argtypes = [vp, vp, vp, vp, vp, vp] + [lg] * 13 + [dbl, dbl, mp, vp, vp, ctypes.c_size_t, vp]
    L.tao_bound_softmax.argtypes = [vp, vp, vp, lg, lg, lg, mp, vp]
    L.tao_bound_norm.argtypes = [ctypes.c_int, vp, vp, vp, vp, dbl, vp, lg, lg, lg, mp, vp]
    L.tao_bound_groupnorm.argtypes = [vp, vp, vp, vp, dbl, vp, lg, lg, lg, lg, mp, vp, ctypes.c_size_t, vp]
    L.tao_groupnorm_workspace_bytes.argtypes = [lg, lg, lg, lg]
    L.tao_groupnorm_workspace_bytes.restype = ctypes.c_size_t
    L.tao_bound_act.argtypes = [ctypes.c_int, vp, vp, vp, vp, lg, mp, vp]
    L.tao_bound_check_act.argtypes = [ctypes.c_int, vp, vp, vp, vp, lg, dbl, dbl, mp, vp, vp, ctypes.c_size_t, vp]
    L.tao_bound_check_norm.argtypes = [ctypes.c_int, vp, vp, vp, vp, dbl, vp, lg, lg, lg, dbl, dbl, mp, vp, vp,
                                       ctypes.c_size_t, vp]
    L.tao_bound_check_rope.argtypes = [vp, vp, vp, vp, vp, lg, lg, lg, lg, ctypes.c_int, dbl, dbl, mp, vp, vp,
                                       ctypes.c_size_t, vp]
    L.tao_bound_rope.argtypes = [vp, vp, vp, vp, lg, lg, lg, lg, ctypes.c_int, mp, vp]
    L.tao_check_and_profile.argtypes = [vp, vp, vp, lg, dbl, dbl, vp, vp, ctypes.c_size_t, vp]
    L.tao_check_and_profile_static.argtypes = [vp, vp, vp, lg, dbl, dbl, vp, vp]
    L.tao_check_workspace_bytes.argtypes = [lg]
    L.tao_bound_check_softmax.argtypes = [vp, vp, vp, lg, lg, lg, dbl, dbl, mp, vp, vp, ctypes.c_size_t, vp]
    L.tao_check_workspace_bytes.restype = ctypes.c_size_t
    L.tao_profile_errors.argtypes = [vp, vp, lg, dbl, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.tao_calibrate_thresholds.argtypes = [vp, lg, dbl, vp, vp, vp, vp, vp]
    L.tao_project_clip.argtypes = [vp, vp, dbl, vp, lg, vp]
    L.tao_project_empirical.argtypes = [vp, vp, dbl, vp, lg, vp, ctypes.c_size_t, vp]
    L.tao_project_workspace_bytes.argtypes = [lg]
    L.tao_project_workspace_bytes.restype = ctypes.c_size_t
    L.tao_profile_workspace_bytes.argtypes = [lg]
    L.tao_profile_workspace_bytes.restype = ctypes.c_size_t
    L.tao_selftest_matrix_core.argtypes = [ctypes.POINTER(ctypes.c_uint), vp, ctypes.c_size_t, vp]
    L.tao_last_hip_error.restype = ctypes.c_int
    L.tao_status_string.argtypes = [ctypes.c_int]
    L.tao_status_string.restype = ctypes.c_char_p
    _lib = L
    return L


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("paper_2510_16028_amd needs a GPU: no CPU fallback exists")
    return torch


def _stream():
    return ctypes.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dev(t, name):
    torch = _torch()
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32):
        raise TypeError("%s must be a float32 CUDA tensor" % name)
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _mref(model):
    return None if model is None else ctypes.byref(model)


def _check(status, where):
    if status != OK:
        raise TaoError(status, where)


def _rows_view(t, name):
    """(rows, cols, ld) of a tensor whose last dimension is contiguous and whose
    leading dimensions collapse to one uniform row stride."""
    if t.dim() == 0:
        raise ValueError("%s: need at least one dimension" % name)
    cols = t.shape[-1]
    if t.dim() == 1:
        return 1, cols, cols
    if cols > 1 and t.stride(-1) != 1:
        raise ValueError("%s: last dimension must be contiguous" % name)
    t2 = t if t.is_contiguous() else None
    if t2 is not None:
        return t.numel() // max(cols, 1), cols, cols
    if t.dim() == 2:
        return t.shape[0], cols, t.stride(0)
    raise ValueError("%s: only 2-D tensors may have a padded row stride" % name)


# ------------------------------------------------------------------ entry points

def tao_default_model():
    m = FpModel()
    lib().tao_default_model(ctypes.byref(m))
    return m


def tao_gamma(k, model=None):
    return lib().tao_gamma(int(k), _mref(model))


def _linear_args(A, W, bias, trans_w, out):
    torch = _torch()
    A = _dev(A, "A"); W = _dev(W, "W"); bias = _dev(bias, "bias")
    if A.dim() not in (2, 3) or W.dim() not in (2, 3):
        raise ValueError("A and W must be 2-D or 3-D")
    for t, nm in ((A, "A"), (W, "W")):
        if t.shape[-1] > 1 and t.stride(-1) != 1:
            raise ValueError("%s: last dimension must be contiguous" % nm)
    batch = A.shape[0] if A.dim() == 3 else 1
    M, K = A.shape[-2], A.shape[-1]
    N = W.shape[-1] if trans_w else W.shape[-2]
    if (W.shape[-2] if trans_w else W.shape[-1]) != K:
        raise ValueError("reduction sizes of A and W differ")
    if W.dim() == 3 and W.shape[0] != batch:
        raise ValueError("batch sizes of A and W differ")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != N or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous [N] tensor")
    shape = (batch, M, N) if A.dim() == 3 else (M, N)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=A.device)
    elif tuple(out.shape) != shape or not out.is_contiguous() or out.dtype != torch.float32:
        raise ValueError("out must be a contiguous float32 tensor of shape %s" % (shape,))
    lda = A.stride(-2) if M > 1 else max(K, 1)
    ldw = W.stride(-2) if W.shape[-2] > 1 else max(W.shape[-1], 1)
    sA = A.stride(0) if A.dim() == 3 and batch > 1 else M * lda
    sW = (W.stride(0) if W.shape[0] > 1 else 0) if W.dim() == 3 else 0
    return A, W, bias, out, (M, N, K, lda, ldw, N, int(bool(trans_w)), batch, sA, sW, M * N)


def tao_bound_linear(A, W, bias=None, trans_w=False, model=None, out=None):
    """tau[..., M, N] for A[..., M, K] and W[N, K] / [B, N, K] (trans_w: [K, N] / [B, K, N])."""
    A, W, bias, out, dims = _linear_args(A, W, bias, trans_w, out)
    rc = lib().tao_bound_linear(_ptr(A), _ptr(W), _ptr(bias), _ptr(out), *dims, _mref(model), _stream())
    _check(rc, "tao_bound_linear")
    return out


def tao_linear_split_workspace_bytes(M, N, K, batch=1, shared_w=True):
    return int(lib().tao_linear_split_workspace_bytes(int(M), int(N), int(K), int(batch), int(bool(shared_w))))


def tao_linear_split_preferred(M, N, K, batch=1):
    _torch()
    return bool(lib().tao_linear_split_preferred(int(M), int(N), int(K), int(batch)))


def tao_selftest_matrix_core_bf16(cases=0):
    torch = _torch()
    rep = ctypes.c_uint(0)
    ws = _scratch(torch.device("cuda", torch.cuda.current_device()), lib().tao_selftest_workspace_bytes(int(cases)))
    _check(lib().tao_selftest_matrix_core_bf16(ctypes.byref(rep), int(cases), _ptr(ws), ws.numel(), _stream()),
           "tao_selftest_matrix_core_bf16")
    return int(rep.value)


def tao_bound_linear_split(A, W, bias=None, trans_w=False, model=None, out=None, ws=None):
    """tao_bound_linear on the BF16 matrix cores (three exact BF16 pieces per operand); same
    arguments, plus an optional scratch tensor."""
    A, W, bias, out, dims = _linear_args(A, W, bias, trans_w, out)
    M, N, K, batch, sW = dims[0], dims[1], dims[2], dims[7], dims[9]
    if ws is None:
        ws = _scratch(A.device, tao_linear_split_workspace_bytes(M, N, K, batch, sW == 0 or batch == 1))
    rc = lib().tao_bound_linear_split(_ptr(A), _ptr(W), _ptr(bias), _ptr(out), *dims, _mref(model),
                                      _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_linear_split")
    return out


def tao_bound_check_linear_in_epilogue(M, N, K, batch=1):
    _torch()
    return bool(lib().tao_bound_check_linear_in_epilogue(int(M), int(N), int(K), int(batch)))


def tao_bound_check_linear_workspace_bytes(M, N, K, batch=1, shared_w=True):
    return int(lib().tao_bound_check_linear_workspace_bytes(int(M), int(N), int(K), int(batch), int(bool(shared_w))))


def tao_bound_check_linear(A, W, bias, y_ref, claimed, trans_w=False, alpha=1.0, eps_rel=1e-12, model=None,
                           tau_out=None, out=None, ws=None, readback=True):
    """The matmul bound of tao_bound_linear_split checked in the kernel's epilogue against
    `claimed` and `y_ref` (contiguous, shaped like the product); tau is stored only into `tau_out`
    if given.  Returns the profile dict (readback=True) or the device buffer."""
    torch = _torch()
    y_ref = _dev(y_ref, "y_ref"); claimed = _dev(claimed, "claimed")
    if tau_out is None:
        # shape checks of A, W, bias against the product's shape, without allocating tau
        A, W, bias, _, dims = _linear_args(A, W, bias, trans_w, y_ref)
    else:
        A, W, bias, tau_out, dims = _linear_args(A, W, bias, trans_w, tau_out)
    M, N, K, batch, sW = dims[0], dims[1], dims[2], dims[7], dims[9]
    shape = (batch, M, N) if A.dim() == 3 else (M, N)
    for t, nm in ((y_ref, "y_ref"), (claimed, "claimed")):
        if tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError("%s must be a contiguous tensor of shape %s" % (nm, shape))
    if out is None:
        out = new_profile_buffer(A.device)
    if ws is None:
        ws = _scratch(A.device, tao_bound_check_linear_workspace_bytes(M, N, K, batch, sW == 0 or batch == 1))
    rc = lib().tao_bound_check_linear(_ptr(A), _ptr(W), _ptr(bias), _ptr(y_ref), _ptr(claimed), _ptr(tau_out),
                                      *dims, float(alpha), float(eps_rel), _mref(model), _ptr(out),
                                      _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_check_linear")
    return read_profile(out) if readback else out


def tao_split_image_bytes(rows, K, batch=1):
    return int(lib().tao_split_image_bytes(int(rows), int(K), int(batch)))


def tao_split_operand(X, trans=False, out=None):
    """The three-piece BF16 image of an operand X [rows, K] or [batch, rows, K] (trans: [.., K, rows]),
    as a uint8 tensor; reusable by every product X takes part in."""
    torch = _torch()
    X = _dev(X, "X")
    if X.dim() not in (2, 3) or (X.shape[-1] > 1 and X.stride(-1) != 1):
        raise ValueError("X must be 2-D or 3-D with a contiguous last dimension")
    batch = X.shape[0] if X.dim() == 3 else 1
    rows, K = (X.shape[-1], X.shape[-2]) if trans else (X.shape[-2], X.shape[-1])
    ld = X.stride(-2) if X.shape[-2] > 1 else max(X.shape[-1], 1)
    stride = X.stride(0) if X.dim() == 3 and batch > 1 else X.shape[-2] * ld
    need = tao_split_image_bytes(rows, K, batch)
    if out is None:
        out = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    rc = lib().tao_split_operand(_ptr(X), rows, K, ld, int(bool(trans)), batch, stride, _ptr(out), out.numel(), _stream())
    _check(rc, "tao_split_operand")
    return out


def tao_bound_linear_images(A_image, W_image, M, N, K, bias=None, batch=1, shared_w=True, model=None, out=None, ws=None):
    """tao_bound_linear_split on prepared images (tao_split_operand); returns tau [M, N] or [batch, M, N]."""
    torch = _torch()
    bias = _dev(bias, "bias")
    shape = (batch, M, N) if batch > 1 else (M, N)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=A_image.device)
    elif out.numel() != batch * M * N or not out.is_contiguous():
        raise ValueError("out must be contiguous with %d elements" % (batch * M * N))
    if ws is None:
        ws = _scratch(A_image.device, lib().tao_linear_images_workspace_bytes(M, N, K, batch))
    rc = lib().tao_bound_linear_images(_ptr(A_image), _ptr(W_image), _ptr(bias), _ptr(out), M, N, K, N, batch, M * N,
                                       int(bool(shared_w)), _mref(model), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_linear_images")
    return out


def tao_bound_check_linear_images(A_image, W_image, M, N, K, y_ref, claimed, bias=None, batch=1, shared_w=True,
                                  alpha=1.0, eps_rel=1e-12, model=None, tau_out=None, out=None, ws=None, readback=True):
    """tao_bound_check_linear on prepared images."""
    y_ref = _dev(y_ref, "y_ref"); claimed = _dev(claimed, "claimed"); bias = _dev(bias, "bias")
    for t, nm in ((y_ref, "y_ref"), (claimed, "claimed"), (tau_out, "tau_out")):
        if t is not None and (t.numel() != batch * M * N or not t.is_contiguous()):
            raise ValueError("%s must be contiguous with %d elements" % (nm, batch * M * N))
    if out is None:
        out = new_profile_buffer(y_ref.device)
    if ws is None:
        ws = _scratch(y_ref.device, lib().tao_check_linear_images_workspace_bytes(M, N, K, batch))
    rc = lib().tao_bound_check_linear_images(_ptr(A_image), _ptr(W_image), _ptr(bias), _ptr(y_ref), _ptr(claimed), _ptr(tau_out),
                                             M, N, K, N, batch, M * N, int(bool(shared_w)), float(alpha), float(eps_rel),
                                             _mref(model), _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_check_linear_images")
    return read_profile(out) if readback else out


def _pair(v, name):
    if isinstance(v, int):
        return v, v
    if len(v) != 2:
        raise ValueError("%s must be an int or a pair" % name)
    return int(v[0]), int(v[1])


def tao_bound_conv2d(x, w, bias=None, stride=1, padding=0, dilation=1, model=None, out=None):
    """tau[B, OH, OW, Cout] for a channels-last input x[B, H, W, C] and filters w[Cout, R, S, C],
    both contiguous (a torch NCHW tensor in channels_last memory format, permuted to
    (0, 2, 3, 1), is such a tensor without a copy)."""
    torch = _torch()
    x = _dev(x, "x"); w = _dev(w, "w"); bias = _dev(bias, "bias")
    if x.dim() != 4 or w.dim() != 4 or not x.is_contiguous() or not w.is_contiguous():
        raise ValueError("x [B, H, W, C] and w [Cout, R, S, C] must be contiguous 4-D tensors")
    B, H, W, C = x.shape
    Cout, R, S, C2 = w.shape
    if C != C2:
        raise ValueError("channel counts of x and w differ")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != Cout or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous [Cout] tensor")
    sh, sw = _pair(stride, "stride"); ph, pw = _pair(padding, "padding"); dh, dw = _pair(dilation, "dilation")
    if min(sh, sw, dh, dw) < 1 or min(ph, pw) < 0 or min(R, S) < 1:
        raise ValueError("bad convolution geometry")
    eh, ew = H + 2 * ph - dh * (R - 1) - 1, W + 2 * pw - dw * (S - 1) - 1
    if eh < 0 or ew < 0:
        raise ValueError("filter larger than the padded input")
    shape = (B, eh // sh + 1, ew // sw + 1, Cout)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    elif tuple(out.shape) != shape or not out.is_contiguous() or out.dtype != torch.float32:
        raise ValueError("out must be a contiguous float32 tensor of shape %s" % (shape,))
    rc = lib().tao_bound_conv2d(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), B, H, W, C, Cout, R, S,
                                sh, sw, ph, pw, dh, dw, _mref(model), _stream())
    _check(rc, "tao_bound_conv2d")
    return out


def _conv_args(x, w, bias, stride, padding, dilation):
    x = _dev(x, "x"); w = _dev(w, "w"); bias = _dev(bias, "bias")
    if x.dim() != 4 or w.dim() != 4 or not x.is_contiguous() or not w.is_contiguous():
        raise ValueError("x [B, H, W, C] and w [Cout, R, S, C] must be contiguous 4-D tensors")
    B, H, W, C = x.shape
    Cout, R, S, C2 = w.shape
    if C != C2:
        raise ValueError("channel counts of x and w differ")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != Cout or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous [Cout] tensor")
    sh, sw = _pair(stride, "stride"); ph, pw = _pair(padding, "padding"); dh, dw = _pair(dilation, "dilation")
    if min(sh, sw, dh, dw) < 1 or min(ph, pw) < 0 or min(R, S) < 1:
        raise ValueError("bad convolution geometry")
    eh, ew = H + 2 * ph - dh * (R - 1) - 1, W + 2 * pw - dw * (S - 1) - 1
    if eh < 0 or ew < 0:
        raise ValueError("filter larger than the padded input")
    geom = (B, H, W, C, Cout, R, S, sh, sw, ph, pw, dh, dw)
    return x, w, bias, geom, (B, eh // sh + 1, ew // sw + 1, Cout)


def tao_conv2d_split_supported(x_shape, w_shape, stride=1, padding=0, dilation=1):
    """Whether tao_bound_conv2d_split / tao_bound_check_conv2d serve this convolution (else: tao_bound_conv2d)."""
    B, H, W, C = x_shape; Cout, R, S, _ = w_shape
    sh, sw = _pair(stride, "stride"); ph, pw = _pair(padding, "padding"); dh, dw = _pair(dilation, "dilation")
    return bool(lib().tao_conv2d_split_supported(B, H, W, C, Cout, R, S, sh, sw, ph, pw, dh, dw))


def tao_bound_conv2d_split(x, w, bias=None, stride=1, padding=0, dilation=1, model=None, out=None, ws=None):
    """tao_bound_conv2d on the BF16 matrix cores (patch matrix gathered and split while loaded)."""
    torch = _torch()
    x, w, bias, geom, shape = _conv_args(x, w, bias, stride, padding, dilation)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    elif tuple(out.shape) != shape or not out.is_contiguous() or out.dtype != torch.float32:
        raise ValueError("out must be a contiguous float32 tensor of shape %s" % (shape,))
    if ws is None:
        ws = _scratch(x.device, lib().tao_conv2d_split_workspace_bytes(*geom, 0))
    rc = lib().tao_bound_conv2d_split(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), *geom, _mref(model), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_conv2d_split")
    return out


def tao_bound_check_conv2d(x, w, bias, y_ref, claimed, stride=1, padding=0, dilation=1, alpha=1.0, eps_rel=1e-12, model=None,
                           tau_out=None, out=None, ws=None, readback=True):
    """The convolution bound of tao_bound_conv2d_split checked on the spot against `claimed` and `y_ref`
    ([B, OH, OW, Cout], contiguous); tau is stored only into `tau_out` if given."""
    x, w, bias, geom, shape = _conv_args(x, w, bias, stride, padding, dilation)
    y_ref = _dev(y_ref, "y_ref"); claimed = _dev(claimed, "claimed")
    n = shape[0] * shape[1] * shape[2] * shape[3]
    for t, nm in ((y_ref, "y_ref"), (claimed, "claimed"), (tau_out, "tau_out")):
        if t is not None and (t.numel() != n or not t.is_contiguous()):
            raise ValueError("%s must be contiguous with %d elements" % (nm, n))
    if out is None:
        out = new_profile_buffer(x.device)
    if ws is None:
        ws = _scratch(x.device, lib().tao_conv2d_split_workspace_bytes(*geom, 1))
    rc = lib().tao_bound_check_conv2d(_ptr(x), _ptr(w), _ptr(bias), _ptr(y_ref), _ptr(claimed), _ptr(tau_out), *geom,
                                      float(alpha), float(eps_rel), _mref(model), _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_check_conv2d")
    return read_profile(out) if readback else out


def tao_bound_softmax(x, y_ref, model=None, out=None):
    torch = _torch()
    x = _dev(x, "x"); y_ref = _dev(y_ref, "y_ref")
    if x.shape != y_ref.shape or x.stride() != y_ref.stride():
        raise ValueError("x and y_ref must have the same shape and strides")
    rows, cols, ld = _rows_view(x, "x")
    if out is None:
        out = torch.empty_strided(x.shape, x.stride(), dtype=torch.float32, device=x.device)
    elif out.shape != x.shape or out.stride() != x.stride():
        raise ValueError("out must match x in shape and strides")
    rc = lib().tao_bound_softmax(_ptr(x), _ptr(y_ref), _ptr(out), rows, cols, ld, _mref(model), _stream())
    _check(rc, "tao_bound_softmax")
    return out


def tao_bound_norm(kind, x, y_ref=None, gamma_or_scale=None, beta_or_shift=None, eps=0.0,
                   model=None, out=None):
    torch = _torch()
    x = _dev(x, "x"); y_ref = _dev(y_ref, "y_ref")
    g = _dev(gamma_or_scale, "gamma_or_scale"); b = _dev(beta_or_shift, "beta_or_shift")
    rows, cols, ld = _rows_view(x, "x")
    reduces = kind in (NORM_SUM, NORM_MEAN)
    for t, nm in ((g, "gamma_or_scale"), (b, "beta_or_shift")):
        if t is not None and (t.dim() != 1 or t.shape[0] != cols or not t.is_contiguous()):
            raise ValueError("%s must be a contiguous [cols] tensor" % nm)
    if reduces:
        if y_ref is not None and (y_ref.numel() != rows or not y_ref.is_contiguous()):
            raise ValueError("y_ref must be a contiguous tensor with one value per row")
        oshape = x.shape[:-1]
        if out is None:
            out = torch.empty(oshape, dtype=torch.float32, device=x.device)
        elif out.numel() != rows or not out.is_contiguous():
            raise ValueError("out must be contiguous with one value per row")
    else:
        if y_ref is not None and (y_ref.shape != x.shape or y_ref.stride() != x.stride()):
            raise ValueError("x and y_ref must have the same shape and strides")
        if out is None:
            out = torch.empty_strided(x.shape, x.stride(), dtype=torch.float32, device=x.device)
        elif out.shape != x.shape or out.stride() != x.stride():
            raise ValueError("out must match x in shape and strides")
    rc = lib().tao_bound_norm(int(kind), _ptr(x), _ptr(y_ref), _ptr(g), _ptr(b), float(eps), _ptr(out),
                              rows, cols, ld, _mref(model), _stream())
    _check(rc, "tao_bound_norm")
    return out


def tao_groupnorm_workspace_bytes(batch, channels, positions, groups):
    return int(lib().tao_groupnorm_workspace_bytes(int(batch), int(channels), int(positions), int(groups)))


def tao_bound_groupnorm(x, y_ref, groups, gamma=None, beta=None, eps=1e-5, model=None, out=None, ws=None):
    """tau like x[N, C, *spatial] (contiguous, channel-major) for GroupNorm with `groups` groups."""
    torch = _torch()
    x = _dev(x, "x"); y_ref = _dev(y_ref, "y_ref"); gamma = _dev(gamma, "gamma"); beta = _dev(beta, "beta")
    if x.dim() < 2 or not x.is_contiguous() or y_ref.shape != x.shape or not y_ref.is_contiguous():
        raise ValueError("x and y_ref must be contiguous [N, C, ...] tensors of one shape")
    N, C = x.shape[0], x.shape[1]
    positions = x.numel() // (N * C) if N * C else 0
    for t, nm in ((gamma, "gamma"), (beta, "beta")):
        if t is not None and (t.dim() != 1 or t.shape[0] != C or not t.is_contiguous()):
            raise ValueError("%s must be a contiguous [C] tensor" % nm)
    if out is None:
        out = torch.empty_like(x)
    elif out.shape != x.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous and shaped like x")
    if ws is None:
        ws = _scratch(x.device, tao_groupnorm_workspace_bytes(N, C, positions, groups))
    rc = lib().tao_bound_groupnorm(_ptr(x), _ptr(y_ref), _ptr(gamma), _ptr(beta), float(eps), _ptr(out),
                                   N, C, positions, int(groups), _mref(model), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_groupnorm")
    return out


def tao_bound_act(kind, x, y_ref, x2=None, model=None, out=None):
    torch = _torch()
    x = _dev(x, "x"); x2 = _dev(x2, "x2"); y_ref = _dev(y_ref, "y_ref")
    for t, nm in ((x, "x"), (x2, "x2"), (y_ref, "y_ref")):
        if t is not None and not t.is_contiguous():
            raise ValueError("%s must be contiguous" % nm)
        if t is not None and t.numel() != y_ref.numel():
            raise ValueError("%s must have as many elements as y_ref" % nm)
    if out is None:
        out = torch.empty_like(y_ref)
    elif out.shape != y_ref.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous and shaped like y_ref")
    rc = lib().tao_bound_act(int(kind), _ptr(x), _ptr(x2), _ptr(y_ref), _ptr(out), y_ref.numel(),
                             _mref(model), _stream())
    _check(rc, "tao_bound_act")
    return out


def tao_bound_rope(x, cos, sin, inner=1, interleaved=False, model=None, out=None):
    """tau like x[..., d] for the rotation of x by the tables cos, sin [npos, d/2]; row r of the
    flattened x uses table row (r // inner) % npos; pairs (j, j + d/2), or (2j, 2j+1) when
    interleaved."""
    torch = _torch()
    x = _dev(x, "x"); cos = _dev(cos, "cos"); sin = _dev(sin, "sin")
    if x.dim() < 1 or not x.is_contiguous() or not cos.is_contiguous() or not sin.is_contiguous():
        raise ValueError("x, cos and sin must be contiguous")
    d = x.shape[-1]
    if cos.dim() != 2 or cos.shape != sin.shape or cos.shape[1] * 2 != d:
        raise ValueError("cos and sin must be [npos, d/2] with d even")
    rows = x.numel() // d if d else 0
    if out is None:
        out = torch.empty_like(x)
    elif out.shape != x.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous and shaped like x")
    rc = lib().tao_bound_rope(_ptr(x), _ptr(cos), _ptr(sin), _ptr(out), rows, d, int(inner), cos.shape[0],
                              int(bool(interleaved)), _mref(model), _stream())
    _check(rc, "tao_bound_rope")
    return out


_ws_cache = {}


def _scratch(device, need):
    """One scratch tensor per (device, stream); calls on one stream are ordered, so sharing is safe."""
    torch = _torch()
    key = (device.index if device.index is not None else torch.cuda.current_device(),
           torch.cuda.current_stream().cuda_stream)
    ws = _ws_cache.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(max(int(need), 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = ws
    return ws


def _workspace(device, n):
    return _scratch(device, lib().tao_check_workspace_bytes(int(n)))


def new_profile_buffer(device):
    """Device buffer able to hold one tao_profile."""
    return _torch().empty(ctypes.sizeof(Profile), dtype=_torch().uint8, device=device)


def read_profile(buf):
    """Copy a tao_profile back from the device (synchronises) and return it as a dict."""
    raw = buf.cpu().numpy().tobytes()
    return Profile.from_buffer_copy(raw).as_dict()


def tao_check_and_profile(claimed, ref, tau, alpha=1.0, eps_rel=1e-12, out=None, ws=None,
                          readback=True):
    """Enqueue the check; with readback=True (default) wait for it and return the profile dict,
    otherwise return the device buffer holding the tao_profile without synchronising."""
    claimed = _dev(claimed, "claimed"); ref = _dev(ref, "ref"); tau = _dev(tau, "tau")
    for t, nm in ((claimed, "claimed"), (ref, "ref"), (tau, "tau")):
        if not t.is_contiguous():
            raise ValueError("%s must be contiguous" % nm)
    n = claimed.numel()
    if ref.numel() != n or tau.numel() != n:
        raise ValueError("claimed, ref and tau must have the same number of elements")
    if out is None:
        out = new_profile_buffer(claimed.device)
    if ws is None:
        ws = _workspace(claimed.device, n)
    rc = lib().tao_check_and_profile(_ptr(claimed), _ptr(ref), _ptr(tau), n, float(alpha),
                                     float(eps_rel), _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_check_and_profile")
    return read_profile(out) if readback else out


STATIC_CHECK_MAX_N = (1 << 36) - 1


def tao_check_and_profile_static(claimed, ref, tau, alpha=1.0, eps_rel=1e-12, out=None, readback=True):
    """tao_check_and_profile through the entry point that allocates nothing (its scratch memory is a
    fixed array inside the library).  `out` must be a buffer from new_profile_buffer when the caller
    may not allocate either."""
    claimed = _dev(claimed, "claimed"); ref = _dev(ref, "ref"); tau = _dev(tau, "tau")
    for t, nm in ((claimed, "claimed"), (ref, "ref"), (tau, "tau")):
        if not t.is_contiguous():
            raise ValueError("%s must be contiguous" % nm)
    n = claimed.numel()
    if ref.numel() != n or tau.numel() != n:
        raise ValueError("claimed, ref and tau must have the same number of elements")
    if out is None:
        out = new_profile_buffer(claimed.device)
    rc = lib().tao_check_and_profile_static(_ptr(claimed), _ptr(ref), _ptr(tau), n, float(alpha),
                                            float(eps_rel), _ptr(out), _stream())
    _check(rc, "tao_check_and_profile_static")
    return read_profile(out) if readback else out


def tao_bound_check_act(kind, x, y_ref, claimed, x2=None, alpha=1.0, eps_rel=1e-12, model=None, out=None,
                        ws=None, readback=True):
    """tao_bound_act checked against `claimed` in one pass, tau never stored."""
    x = _dev(x, "x"); x2 = _dev(x2, "x2"); y_ref = _dev(y_ref, "y_ref"); claimed = _dev(claimed, "claimed")
    for t, nm in ((x, "x"), (x2, "x2"), (y_ref, "y_ref"), (claimed, "claimed")):
        if t is not None and (not t.is_contiguous() or t.numel() != y_ref.numel()):
            raise ValueError("%s must be contiguous and sized like y_ref" % nm)
    n = y_ref.numel()
    if out is None:
        out = new_profile_buffer(y_ref.device)
    if ws is None:
        ws = _workspace(y_ref.device, n)
    rc = lib().tao_bound_check_act(int(kind), _ptr(x), _ptr(x2), _ptr(y_ref), _ptr(claimed), n, float(alpha),
                                   float(eps_rel), _mref(model), _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_check_act")
    return read_profile(out) if readback else out


def tao_bound_check_norm(kind, x, y_ref, claimed, g=None, b=None, eps=0.0, alpha=1.0, eps_rel=1e-12, model=None,
                         out=None, ws=None, readback=True):
    """tao_bound_norm (LayerNorm or RMSNorm) checked against `claimed` in one pass, tau never stored."""
    x = _dev(x, "x"); y_ref = _dev(y_ref, "y_ref"); claimed = _dev(claimed, "claimed"); g = _dev(g, "g"); b = _dev(b, "b")
    for t, nm in ((y_ref, "y_ref"), (claimed, "claimed")):
        if t.shape != x.shape or t.stride() != x.stride():
            raise ValueError("%s must have the shape and strides of x" % nm)
    rows, cols, ld = _rows_view(x, "x")
    for t, nm in ((g, "g"), (b, "b")):
        if t is not None and (t.dim() != 1 or t.shape[0] != cols or not t.is_contiguous()):
            raise ValueError("%s must be a contiguous [cols] tensor" % nm)
    if out is None:
        out = new_profile_buffer(x.device)
    if ws is None:
        ws = _workspace(x.device, rows * cols)
    rc = lib().tao_bound_check_norm(int(kind), _ptr(x), _ptr(y_ref), _ptr(g), _ptr(b), float(eps), _ptr(claimed),
                                    rows, cols, ld, float(alpha), float(eps_rel), _mref(model), _ptr(out),
                                    _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_check_norm")
    return read_profile(out) if readback else out


def tao_bound_check_rope(x, cos, sin, y_ref, claimed, inner=1, interleaved=False, alpha=1.0, eps_rel=1e-12,
                         model=None, out=None, ws=None, readback=True):
    """tao_bound_rope checked against `claimed` in one pass, tau never stored."""
    x = _dev(x, "x"); cos = _dev(cos, "cos"); sin = _dev(sin, "sin")
    y_ref = _dev(y_ref, "y_ref"); claimed = _dev(claimed, "claimed")
    if x.dim() < 1 or not x.is_contiguous() or not cos.is_contiguous() or not sin.is_contiguous():
        raise ValueError("x, cos and sin must be contiguous")
    d = x.shape[-1]
    if cos.dim() != 2 or cos.shape != sin.shape or cos.shape[1] * 2 != d:
        raise ValueError("cos and sin must be [npos, d/2] tables")
    for t, nm in ((y_ref, "y_ref"), (claimed, "claimed")):
        if t.shape != x.shape or not t.is_contiguous():
            raise ValueError("%s must be contiguous and shaped like x" % nm)
    rows = x.numel() // max(d, 1)
    if out is None:
        out = new_profile_buffer(x.device)
    if ws is None:
        ws = _workspace(x.device, x.numel())
    rc = lib().tao_bound_check_rope(_ptr(x), _ptr(cos), _ptr(sin), _ptr(y_ref), _ptr(claimed), rows, d, int(inner),
                                    cos.shape[0], int(bool(interleaved)), float(alpha), float(eps_rel), _mref(model),
                                    _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_check_rope")
    return read_profile(out) if readback else out


def tao_bound_check_softmax(x, y_ref, claimed, alpha=1.0, eps_rel=1e-12, model=None, out=None, ws=None,
                            readback=True):
    """The softmax bound checked against `claimed` in one pass; same result as tao_bound_softmax
    followed by tao_check_and_profile(claimed, y_ref, tau), without a stored tau."""
    x = _dev(x, "x"); y_ref = _dev(y_ref, "y_ref"); claimed = _dev(claimed, "claimed")
    if x.shape != y_ref.shape or x.stride() != y_ref.stride() or claimed.shape != x.shape or claimed.stride() != x.stride():
        raise ValueError("x, y_ref and claimed must have the same shape and strides")
    rows, cols, ld = _rows_view(x, "x")
    if out is None:
        out = new_profile_buffer(x.device)
    if ws is None:
        ws = _workspace(x.device, rows * cols)
    rc = lib().tao_bound_check_softmax(_ptr(x), _ptr(y_ref), _ptr(claimed), rows, cols, ld, float(alpha),
                                       float(eps_rel), _mref(model), _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_bound_check_softmax")
    return read_profile(out) if readback else out


def tao_profile_errors(claimed, ref, eps_rel=1e-12, thr_abs=None, thr_rel=None, out=None, ws=None,
                       readback=True):
    """Absolute / relative error profiles on the 22-point grid and the selection statistic.
    thr_abs, thr_rel: float32 CUDA tensors of 22 thresholds (both or neither)."""
    torch = _torch()
    claimed = _dev(claimed, "claimed"); ref = _dev(ref, "ref")
    thr_abs = _dev(thr_abs, "thr_abs"); thr_rel = _dev(thr_rel, "thr_rel")
    for t, nm in ((claimed, "claimed"), (ref, "ref")):
        if not t.is_contiguous():
            raise ValueError("%s must be contiguous" % nm)
    n = claimed.numel()
    if ref.numel() != n:
        raise ValueError("claimed and ref must have the same number of elements")
    if (thr_abs is None) != (thr_rel is None):
        raise ValueError("thr_abs and thr_rel come together")
    for t, nm in ((thr_abs, "thr_abs"), (thr_rel, "thr_rel")):
        if t is not None and (t.numel() != NGRID or not t.is_contiguous()):
            raise ValueError("%s must be a contiguous tensor of %d thresholds" % (nm, NGRID))
    if out is None:
        out = torch.empty(ctypes.sizeof(ErrorProfile), dtype=torch.uint8, device=claimed.device)
    need = lib().tao_profile_workspace_bytes(int(n))
    if ws is None:
        key = ("errors", claimed.device.index if claimed.device.index is not None else torch.cuda.current_device(),
               torch.cuda.current_stream().cuda_stream)
        ws = _ws_cache.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=claimed.device)
            _ws_cache[key] = ws
    rc = lib().tao_profile_errors(_ptr(claimed), _ptr(ref), n, float(eps_rel), _ptr(thr_abs), _ptr(thr_rel),
                                  _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "tao_profile_errors")
    if not readback:
        return out
    return ErrorProfile.from_buffer_copy(out.cpu().numpy().tobytes()).as_dict()


def tao_calibrate_thresholds(profiles, alpha=3.0):
    """profiles: uint8 CUDA tensor holding `count` consecutive tao_error_profile structs (the
    `out` buffers of tao_profile_errors, e.g. rows of one [count, sizeof] tensor).
    Returns (env_abs, env_rel, thr_abs, thr_rel) as float32 CUDA tensors of 22 values."""
    torch = _torch()
    size = ctypes.sizeof(ErrorProfile)
    if not (isinstance(profiles, torch.Tensor) and profiles.is_cuda and profiles.dtype == torch.uint8
            and profiles.is_contiguous() and profiles.numel() % size == 0):
        raise TypeError("profiles must be a contiguous uint8 CUDA tensor of whole tao_error_profile structs")
    count = profiles.numel() // size
    outs = [torch.empty(NGRID, dtype=torch.float32, device=profiles.device) for _ in range(4)]
    rc = lib().tao_calibrate_thresholds(_ptr(profiles), count, float(alpha), *[_ptr(o) for o in outs], _stream())
    _check(rc, "tao_calibrate_thresholds")
    return tuple(outs)


def tao_project_clip(delta, tau, alpha=1.0, out=None):
    """clip(delta, -alpha tau, alpha tau) (Sec. 4.4 (i)); float32 CUDA tensors of one shape."""
    torch = _torch()
    delta = _dev(delta, "delta"); tau = _dev(tau, "tau")
    if delta.shape != tau.shape or not (delta.is_contiguous() and tau.is_contiguous()):
        raise ValueError("delta and tau must be contiguous tensors of one shape")
    if out is None:
        out = torch.empty_like(delta)
    elif _dev(out, "out").shape != delta.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous and shaped like delta")
    _check(lib().tao_project_clip(_ptr(delta), _ptr(tau), float(alpha), _ptr(out), delta.numel(), _stream()),
           "tao_project_clip")
    return out


def tao_project_workspace_bytes(n):
    return lib().tao_project_workspace_bytes(int(n))


def tao_project_empirical(delta, thr_abs, alpha=1.0, out=None, ws=None):
    """Order-statistic projection onto the empirical admissible set (Sec. 4.4 (ii)).
    delta: contiguous float32 CUDA tensor; thr_abs: 22 float32 thresholds on the same device."""
    torch = _torch()
    delta = _dev(delta, "delta"); thr_abs = _dev(thr_abs, "thr_abs")
    if not delta.is_contiguous() or thr_abs.numel() != NGRID or not thr_abs.is_contiguous():
        raise ValueError("delta must be contiguous and thr_abs hold %d contiguous values" % NGRID)
    if out is None:
        out = torch.empty_like(delta)
    elif _dev(out, "out").shape != delta.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous and shaped like delta")
    n = delta.numel()
    need = lib().tao_project_workspace_bytes(n)
    if ws is None:
        ws = _scratch(delta.device, need)
    _check(lib().tao_project_empirical(_ptr(delta), _ptr(thr_abs), float(alpha), _ptr(out), n,
                                       _ptr(ws), ws.numel(), _stream()), "tao_project_empirical")
    return out


def tao_profile_workspace_bytes(n):
    return lib().tao_profile_workspace_bytes(int(n))


def tao_check_workspace_bytes(n):
    return lib().tao_check_workspace_bytes(int(n))


def tao_selftest_matrix_core():
    """Bit mask: 1 accumulation rounds to nearest-even, 2 subnormals kept, 4 chain within gamma_6."""
    torch = _torch()
    rep = ctypes.c_uint(0)
    ws = _scratch(torch.device("cuda", torch.cuda.current_device()), lib().tao_selftest_workspace_bytes(0))
    _check(lib().tao_selftest_matrix_core(ctypes.byref(rep), _ptr(ws), ws.numel(), _stream()), "tao_selftest_matrix_core")
    return int(rep.value)
