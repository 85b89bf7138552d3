"""Host-side tests of the C ABI that need no GPU: the shared library loads, exports every
function include/tao.h declares, and rejects bad arguments with the documented status
codes before anything is enqueued."""
import ctypes
import math
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tao():
    import paper_2510_16028_amd as t
    if not os.path.exists(t.LIB_PATH):
        from paper_2510_16028_amd import build
        build.build()
    t.lib()
    return t


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "tao.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tao_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_function(tao):
    names = _declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(tao.lib(), n), "libtao.so does not export %s" % n
    assert set(names) == set(tao.EXPORTS)


def test_struct_layouts_match_the_header(tao):
    assert ctypes.sizeof(tao.Profile) == 8 * 3 + 4 * 10 + 8 * 2048
    assert tao.Profile.hist.offset == 64
    assert ctypes.sizeof(tao.FpModel) == 104 and tao.FpModel.c_log.offset == 64
    assert ctypes.sizeof(tao.ErrorProfile) == 8 * 2 + 4 * 2 + 4 * 22 * 4 + 8 + 4 * 2 + 8 * 2048 * 2
    assert tao.ErrorProfile.p_max.offset % 8 == 0 and tao.ErrorProfile.hist_abs.offset % 8 == 0
    assert tao.GRID_PERCENT == [1, 5, 10, 15, 20, 25, 30, 35, 40, 45, 50, 55, 60, 65, 70, 75, 80, 85, 90,
                                95, 99, 100]
    m = tao.tao_default_model()
    assert (m.u, m.mode, m.lam, m.c_exp, m.c_erf, m.c_rsqrt, m.c_div, m.flags) == \
        (2.0 ** -24, 0, 4.0, 2.0, 2.0, 2.0, 2.0, 0)
    assert (m.c_log, m.c_sin, m.c_cos, m.c_tanh, m.c_pow) == (2.0, 4.0, 4.0, 4.0, 8.0)


def test_host_gamma(tao):
    assert tao.tao_gamma(0) == 0.0
    g = tao.tao_gamma(256)
    assert 1 / 65535 <= g <= (1 / 65535) * (1 + 1e-14)
    assert math.isnan(tao.tao_gamma(2 ** 24))
    gp = tao.tao_gamma(256, tao.FpModel(mode=1))
    assert abs(gp - 3.8147e-6) < 1e-9
    assert math.isnan(tao.tao_gamma(10, tao.FpModel(mode=7)))


def test_argument_validation_without_a_gpu(tao):
    L = tao.lib()
    p = ctypes.c_void_p(0x1000)        # aligned dummy pointer; never dereferenced on these paths
    odd = ctypes.c_void_p(0x1002)
    nul = ctypes.c_void_p(0)
    # softmax
    assert L.tao_bound_softmax(p, p, p, -1, 4, 4, None, None) == tao.ERR_SHAPE
    assert L.tao_bound_softmax(p, p, p, 4, 8, 4, None, None) == tao.ERR_SHAPE          # ld < cols
    assert L.tao_bound_softmax(nul, p, p, 4, 4, 4, None, None) == tao.ERR_NULL
    assert L.tao_bound_softmax(odd, p, p, 4, 4, 4, None, None) == tao.ERR_ALIGN
    assert L.tao_bound_softmax(p, p, p, 4, 2 ** 24 + 2, 2 ** 24 + 2, None, None) == tao.ERR_K_RANGE
    assert L.tao_bound_softmax(nul, nul, nul, 0, 4, 4, None, None) == tao.OK             # empty: no-op
    bad = tao.FpModel(u=0.5)
    assert L.tao_bound_softmax(p, p, p, 4, 4, 4, ctypes.byref(bad), None) == tao.ERR_MODEL
    assert L.tao_bound_softmax(p, p, p, 4, 4, 4, ctypes.byref(tao.FpModel(flags=8)), None) == tao.ERR_MODEL     # unknown flag bit
    # norm
    assert L.tao_bound_norm(9, p, p, p, p, 1e-5, p, 4, 4, 4, None, None) == tao.ERR_KIND
    assert L.tao_bound_norm(0, nul, p, p, p, 1e-5, p, 4, 4, 4, None, None) == tao.ERR_NULL   # x required (y_ref may be NULL)
    assert L.tao_bound_norm(0, p, nul, p, odd, 1e-5, p, 4, 4, 4, None, None) == tao.ERR_ALIGN  # the shift enters the bound without y_ref
    assert L.tao_bound_norm(2, p, p, nul, p, 0.0, p, 4, 4, 4, None, None) == tao.ERR_NULL    # scale required
    assert L.tao_bound_norm(0, p, p, p, p, -1.0, p, 4, 4, 4, None, None) == tao.ERR_SHAPE
    # groupnorm: (eps, tau, batch, channels, positions, groups)
    gn = lambda *a: L.tao_bound_groupnorm(*a, None, nul, 0, None)
    assert gn(p, p, p, p, 1e-5, p, 2, 10, 16, 4) == tao.ERR_SHAPE    # 10 % 4
    assert gn(p, p, p, p, 1e-5, p, 2, 8, 16, 0) == tao.ERR_SHAPE
    assert gn(p, p, p, p, -1.0, p, 2, 8, 16, 4) == tao.ERR_SHAPE
    assert gn(p, p, p, p, 1e-5, p, 2, 8, 2 ** 31, 4) == tao.ERR_SHAPE
    assert gn(p, p, p, p, 1e-5, p, 2, 8, 2 ** 24, 4) == tao.ERR_K_RANGE
    assert gn(p, nul, p, p, 1e-5, p, 2, 8, 16, 4) == tao.ERR_NULL
    assert gn(odd, p, p, p, 1e-5, p, 2, 8, 16, 4) == tao.ERR_ALIGN
    assert gn(nul, nul, nul, nul, 1e-5, nul, 0, 8, 16, 4) == tao.OK
    assert gn(p, p, p, p, 1e-5, p, 2, 8, 8192, 4) == tao.ERR_WORKSPACE       # rows of 16384 need scratch
    assert L.tao_groupnorm_workspace_bytes(2, 8, 8192, 4) == 2 * 4 * 2 * 4 * 8
    assert L.tao_groupnorm_workspace_bytes(2, 8, 4096, 4) == 0 and L.tao_groupnorm_workspace_bytes(2, 9, 8192, 4) == 0
    # act
    assert L.tao_bound_act(18, p, p, p, p, 4, None, None) == tao.ERR_KIND
    assert L.tao_bound_act(-1, p, p, p, p, 4, None, None) == tao.ERR_KIND
    assert L.tao_bound_act(17, nul, nul, p, p, 4, None, None) == tao.ERR_NULL                # tanh-form GELU needs x
    assert L.tao_bound_act(11, p, p, p, p, 4, ctypes.byref(tao.FpModel(c_log=-1.0)), None) == tao.ERR_MODEL
    # rope: (rows, d, inner, npos, interleaved)
    assert L.tao_bound_rope(p, p, p, p, 4, 7, 1, 1, 0, None, None) == tao.ERR_SHAPE          # odd d
    assert L.tao_bound_rope(p, p, p, p, 4, 8, 0, 1, 0, None, None) == tao.ERR_SHAPE
    assert L.tao_bound_rope(p, p, p, p, 4, 8, 1, 0, 0, None, None) == tao.ERR_SHAPE
    assert L.tao_bound_rope(p, nul, p, p, 4, 8, 1, 1, 0, None, None) == tao.ERR_NULL
    assert L.tao_bound_rope(p, p, odd, p, 4, 8, 1, 1, 0, None, None) == tao.ERR_ALIGN
    assert L.tao_bound_rope(nul, nul, nul, nul, 0, 8, 1, 1, 0, None, None) == tao.OK
    assert L.tao_bound_act(0, nul, nul, p, p, 4, None, None) == tao.ERR_NULL                 # GELU needs x
    assert L.tao_bound_act(1, nul, nul, p, p, -4, None, None) == tao.ERR_SHAPE
    assert L.tao_bound_act(1, nul, nul, nul, nul, 0, None, None) == tao.OK
    cneed = L.tao_check_workspace_bytes(100)
    wsp = ctypes.c_void_p(0x100000)
    assert L.tao_bound_check_act(1, nul, nul, p, p, 10, 1.0, 0.0, None, nul, wsp, cneed, None) == tao.ERR_NULL
    assert L.tao_bound_check_act(1, nul, nul, p, p, 10, 1.0, 0.0, None, p, nul, cneed, None) == tao.ERR_WORKSPACE
    assert L.tao_bound_check_act(1, nul, nul, p, p, 10, 1.0, 0.0, None, p, wsp, cneed - 1, None) == tao.ERR_WORKSPACE
    assert L.tao_bound_check_act(1, nul, nul, p, nul, 10, 1.0, 0.0, None, p, wsp, cneed, None) == tao.ERR_NULL
    assert L.tao_bound_check_act(0, nul, nul, p, p, 10, 1.0, 0.0, None, p, wsp, cneed, None) == tao.ERR_NULL   # GELU needs x
    assert L.tao_bound_check_act(18, nul, nul, p, p, 10, 1.0, 0.0, None, p, wsp, cneed, None) == tao.ERR_KIND
    assert L.tao_bound_check_act(1, nul, nul, p, p, -1, 1.0, 0.0, None, p, wsp, cneed, None) == tao.ERR_SHAPE
    assert L.tao_bound_check_act(1, nul, nul, p, p, 10, -1.0, 0.0, None, p, wsp, cneed, None) == tao.ERR_SHAPE
    assert L.tao_bound_check_act(1, nul, nul, p, odd, 10, 1.0, 0.0, None, p, wsp, cneed, None) == tao.ERR_ALIGN
    fr = lambda x_, y_, c_, rows, d, inner, npos, a, e, o, w_, wn: L.tao_bound_check_rope(x_, p, p, y_, c_, rows, d, inner, npos, 0, a, e, None, o, w_, wn, None)
    assert fr(p, p, p, 4, 7, 1, 1, 1.0, 0.0, p, wsp, cneed) == tao.ERR_SHAPE          # odd d
    assert fr(p, p, p, 4, 8, 0, 1, 1.0, 0.0, p, wsp, cneed) == tao.ERR_SHAPE
    assert fr(p, p, p, 4, 8, 1, 1, 1.0, -1.0, p, wsp, cneed) == tao.ERR_SHAPE
    assert fr(p, nul, p, 4, 8, 1, 1, 1.0, 0.0, p, wsp, cneed) == tao.ERR_NULL
    assert fr(p, p, p, 4, 8, 1, 1, 1.0, 0.0, nul, wsp, cneed) == tao.ERR_NULL
    assert fr(p, p, odd, 4, 8, 1, 1, 1.0, 0.0, p, wsp, cneed) == tao.ERR_ALIGN
    assert fr(p, p, p, 4, 8, 1, 1, 1.0, 0.0, p, wsp, cneed - 1) == tao.ERR_WORKSPACE
    fn = lambda kind, x_, y_, c_, rows, cols, ld, a, e, o, w_, wn: L.tao_bound_check_norm(kind, x_, y_, p, p, 1e-5, c_, rows, cols, ld, a, e, None, o, w_, wn, None)
    assert fn(2, p, p, p, 4, 8, 8, 1.0, 0.0, p, wsp, cneed) == tao.ERR_KIND              # only LayerNorm and RMSNorm
    assert fn(0, p, p, p, 4, 8, 4, 1.0, 0.0, p, wsp, cneed) == tao.ERR_SHAPE             # ld < cols
    assert fn(1, p, p, p, 4, 8, 8, 1.0, float("nan"), p, wsp, cneed) == tao.ERR_SHAPE
    assert fn(1, p, nul, p, 4, 8, 8, 1.0, 0.0, p, wsp, cneed) == tao.ERR_NULL
    assert fn(1, p, p, p, 4, 8, 8, 1.0, 0.0, nul, wsp, cneed) == tao.ERR_NULL
    assert fn(0, p, p, odd, 4, 8, 8, 1.0, 0.0, p, wsp, cneed) == tao.ERR_ALIGN
    assert fn(0, p, p, p, 4, 8, 8, 1.0, 0.0, p, nul, cneed) == tao.ERR_WORKSPACE
    assert fn(0, p, p, p, 4, 2 ** 24 + 2, 2 ** 24 + 2, 1.0, 0.0, p, wsp, cneed) == tao.ERR_K_RANGE
    # linear
    args = lambda M, N, K, lda, ldw, ldt, tw=0, batch=1: (M, N, K, lda, ldw, ldt, tw, batch, 0, 0, 0)
    assert L.tao_bound_linear(p, p, nul, p, *args(4, 4, 8, 4, 8, 4), None, None) == tao.ERR_SHAPE   # lda < K
    assert L.tao_bound_linear(p, p, nul, p, *args(4, 4, 8, 8, 8, 2), None, None) == tao.ERR_SHAPE   # ldt < N
    assert L.tao_bound_linear(p, p, nul, p, *args(4, 4, 8, 8, 2, 4, 1), None, None) == tao.ERR_SHAPE  # trans: ldw < N
    assert L.tao_bound_linear(p, p, nul, p, *args(-1, 4, 8, 8, 8, 4), None, None) == tao.ERR_SHAPE
    K = 2 ** 24
    assert L.tao_bound_linear(p, p, nul, p, *args(4, 4, K, K, K, 4), None, None) == tao.ERR_K_RANGE
    assert L.tao_bound_linear(nul, p, nul, p, *args(4, 4, 8, 8, 8, 4), None, None) == tao.ERR_NULL
    assert L.tao_bound_linear(p, odd, nul, p, *args(4, 4, 8, 8, 8, 4), None, None) == tao.ERR_ALIGN
    assert L.tao_bound_linear(nul, nul, nul, nul, *args(0, 4, 8, 8, 8, 4), None, None) == tao.OK
    # the same through the BF16 path: needs a workspace
    wsb = L.tao_linear_split_workspace_bytes(4, 4, 8, 1, 1)
    assert wsb == 2 * (24576 + 512) and L.tao_linear_split_workspace_bytes(0, 4, 8, 1, 1) == 0
    assert L.tao_linear_split_workspace_bytes(300, 129, 33, 2, 0) == 2 * (3 + 2) * 2 * 24576 + 2 * 512
    # fewer tiles than compute units (256 assumed without a device) and a long reduction: the reduction is
    # cut into parts whose binary64 partial sums follow the operands in the workspace
    operands = (4096 // 32) * (16 + 8) * 24576 + 2 * 512       # two images, 512 bytes of slack each
    assert L.tao_linear_split_workspace_bytes(2048, 1024, 4096, 1, 1) == (operands + 255) // 256 * 256 + 2 * 2048 * 1024 * 8
    assert L.tao_linear_split_workspace_bytes(2048, 4096, 4096, 1, 1) == (4096 // 32) * (16 + 32) * 24576 + 2 * 512   # 512 tiles: one part
    operands = (256 // 32) * (16 + 8) * 24576 + 2 * 512          # 8 groups: two parts of four
    assert L.tao_linear_split_workspace_bytes(2048, 1024, 256, 1, 1) == (operands + 255) // 256 * 256 + 2 * 2048 * 1024 * 8
    assert L.tao_linear_split_workspace_bytes(2048, 1024, 96, 1, 1) == (96 // 32) * (16 + 8) * 24576 + 2 * 512       # too short to cut
    L.tao_linear_split_preferred.restype = ctypes.c_int
    assert L.tao_linear_split_preferred(2048, 1024, 4096, 1) == 1 and L.tao_linear_split_preferred(2048, 4096, 4096, 1) == 1
    assert L.tao_linear_split_preferred(8192, 128, 2048, 8) == 1 and L.tao_linear_split_preferred(128, 1024, 1024, 1) == 0
    assert L.tao_linear_split_preferred(8192, 128, 1024, 8) == 0 and L.tao_linear_split_preferred(2048, 128, 2048, 8) == 0
    assert L.tao_bound_check_linear_in_epilogue(2048, 4096, 4096, 1) == 1 and L.tao_bound_check_linear_in_epilogue(8192, 2048, 128, 8) == 0
    assert L.tao_bound_check_linear_in_epilogue(64, 64, 96, 1) == 0 and L.tao_bound_check_linear_in_epilogue(64, 64, 1025, 1) == 1
    assert L.tao_bound_check_linear_in_epilogue(64, 64, 1024, 1) == 1       # cut into parts: checked by the pass that adds them
    big = ctypes.c_void_p(0x100000)
    assert L.tao_bound_linear_split(p, p, nul, p, *args(4, 4, 8, 4, 8, 4), None, big, wsb, None) == tao.ERR_SHAPE
    assert L.tao_bound_linear_split(p, p, nul, p, *args(4, 4, 8, 8, 8, 4), None, nul, wsb, None) == tao.ERR_WORKSPACE
    assert L.tao_bound_linear_split(p, p, nul, p, *args(4, 4, 8, 8, 8, 4), None, big, wsb - 1, None) == tao.ERR_WORKSPACE
    assert L.tao_bound_linear_split(p, p, nul, p, *args(4, 4, 8, 8, 8, 4), None, ctypes.c_void_p(0x100010), wsb, None) == tao.ERR_WORKSPACE
    assert L.tao_bound_linear_split(nul, p, nul, p, *args(4, 4, 8, 8, 8, 4), None, big, wsb, None) == tao.ERR_NULL
    assert L.tao_bound_linear_split(p, p, nul, p, *args(4, 4, K, K, K, 4), None, big, wsb, None) == tao.ERR_K_RANGE
    assert L.tao_bound_linear_split(nul, nul, nul, nul, *args(0, 4, 8, 8, 8, 4), None, nul, 0, None) == tao.OK
    # ... and with the check fused into the epilogue
    cwb = L.tao_bound_check_linear_workspace_bytes(4, 4, 8, 1, 1)
    # (a reduction up to 1024 long: room for the stored bound, 4 x 4 x 4 bytes rounded to 256)
    assert cwb == (wsb + 255) // 256 * 256 + L.tao_check_workspace_bytes(16) + 256
    wsb_long = L.tao_linear_split_workspace_bytes(4, 4, 2048, 1, 1)
    assert L.tao_bound_check_linear_workspace_bytes(4, 4, 2048, 1, 1) == (wsb_long + 255) // 256 * 256 + L.tao_check_workspace_bytes(16)
    fc = lambda a, w, y, c, t, dims, alpha, out, wsp, wsn: L.tao_bound_check_linear(a, w, nul, y, c, t, *dims, alpha, 0.0, None, out, wsp, wsn, None)
    ok = args(4, 4, 8, 8, 8, 4)
    assert fc(p, p, p, p, nul, args(4, 4, 8, 4, 8, 4), 1.0, p, big, cwb) == tao.ERR_SHAPE        # lda < K
    assert fc(p, p, p, p, nul, args(4, 4, 8, 8, 8, 2), 1.0, p, big, cwb) == tao.ERR_SHAPE        # ldy < N
    assert fc(p, p, p, p, nul, ok, -1.0, p, big, cwb) == tao.ERR_SHAPE
    assert fc(p, p, p, p, nul, ok, 1.0, nul, big, cwb) == tao.ERR_NULL                           # no result buffer
    assert fc(p, p, nul, p, nul, ok, 1.0, p, big, cwb) == tao.ERR_NULL
    assert fc(p, p, p, nul, nul, ok, 1.0, p, big, cwb) == tao.ERR_NULL
    assert fc(nul, p, p, p, nul, ok, 1.0, p, big, cwb) == tao.ERR_NULL
    assert fc(p, p, odd, p, nul, ok, 1.0, p, big, cwb) == tao.ERR_ALIGN
    assert fc(p, p, p, p, nul, ok, 1.0, p, nul, cwb) == tao.ERR_WORKSPACE
    assert fc(p, p, p, p, nul, ok, 1.0, p, big, cwb - 1) == tao.ERR_WORKSPACE
    assert fc(p, p, p, p, nul, args(4, 4, K, K, K, 4), 1.0, p, big, 1 << 40) == tao.ERR_K_RANGE
    assert fc(p, p, p, p, nul, args(1 << 18, 1 << 18, 8, 8, 8, 1 << 18), 1.0, p, big, 1 << 50) == tao.ERR_SHAPE   # 2^36 outputs
    # prepared operands: the image of an operand, and the products on two images
    L.tao_split_image_bytes.restype = ctypes.c_size_t
    ib = L.tao_split_image_bytes(4, 8, 1)
    assert ib == 24576 + 512 and L.tao_split_image_bytes(300, 33, 2) == 3 * 2 * 2 * 24576 + 512 and L.tao_split_image_bytes(0, 8, 1) == 0
    so = lambda src, rows, K_, ld, tr, img, nbytes: L.tao_split_operand(src, rows, K_, ld, tr, 1, 0, img, nbytes, None)
    assert so(p, 4, 8, 4, 0, big, ib) == tao.ERR_SHAPE                 # ld < K
    assert so(p, 4, 8, 2, 1, big, ib) == tao.ERR_SHAPE                 # transposed: ld < rows
    assert so(nul, 4, 8, 8, 0, big, ib) == tao.ERR_NULL
    assert so(odd, 4, 8, 8, 0, big, ib) == tao.ERR_ALIGN
    assert so(p, 4, 8, 8, 0, nul, ib) == tao.ERR_WORKSPACE
    assert so(p, 4, 8, 8, 0, big, ib - 1) == tao.ERR_WORKSPACE
    assert so(p, 4, 8, 8, 0, ctypes.c_void_p(0x100010), ib) == tao.ERR_WORKSPACE
    assert so(nul, 0, 8, 8, 0, nul, 0) == tao.OK
    L.tao_linear_images_workspace_bytes.restype = ctypes.c_size_t
    L.tao_check_linear_images_workspace_bytes.restype = ctypes.c_size_t
    assert L.tao_linear_images_workspace_bytes(2048, 4096, 4096, 1) == 0
    assert L.tao_linear_images_workspace_bytes(2048, 1024, 4096, 1) == 2 * 2048 * 1024 * 8
    assert L.tao_check_linear_images_workspace_bytes(4, 4, 8, 1) == L.tao_check_workspace_bytes(16) + 256
    fi = lambda a, w, t, M, N, K_, ldt, wsp, wsn: L.tao_bound_linear_images(a, w, nul, t, M, N, K_, ldt, 1, 0, 1, None, wsp, wsn, None)
    assert fi(big, big, p, 4, 4, 8, 2, nul, 0) == tao.ERR_SHAPE        # ldt < N
    assert fi(big, big, p, 4, 4, K, 4, nul, 0) == tao.ERR_K_RANGE
    assert fi(nul, big, p, 4, 4, 8, 4, nul, 0) == tao.ERR_NULL
    assert fi(big, big, nul, 4, 4, 8, 4, nul, 0) == tao.ERR_NULL
    assert fi(ctypes.c_void_p(0x100010), big, p, 4, 4, 8, 4, nul, 0) == tao.ERR_ALIGN
    assert fi(big, big, p, 2048, 1024, 4096, 1024, nul, 0) == tao.ERR_WORKSPACE      # parts: needs the partial sums
    assert fi(nul, nul, nul, 0, 4, 8, 4, nul, 0) == tao.OK
    ciw = L.tao_check_linear_images_workspace_bytes(4, 4, 8, 1)
    fci = lambda a, w, y, c, o, wsp, wsn: L.tao_bound_check_linear_images(a, w, nul, y, c, nul, 4, 4, 8, 4, 1, 0, 1, 1.0, 0.0, None, o, wsp, wsn, None)
    assert fci(big, big, p, p, nul, big, ciw) == tao.ERR_NULL
    assert fci(big, big, nul, p, p, big, ciw) == tao.ERR_NULL
    assert fci(big, big, p, p, p, big, ciw - 1) == tao.ERR_WORKSPACE
    assert fci(big, big, p, p, p, nul, ciw) == tao.ERR_WORKSPACE
    # conv2d: (batch, H, W, C, Cout, R, S, stride h/w, pad h/w, dilation h/w)
    cargs = lambda B=1, H=8, W=8, C=4, Co=4, R=3, S=3, sh=1, sw=1, ph=1, pw=1, dh=1, dw=1: \
        (B, H, W, C, Co, R, S, sh, sw, ph, pw, dh, dw)
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(sh=0), None, None) == tao.ERR_SHAPE
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(dw=0), None, None) == tao.ERR_SHAPE
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(ph=-1), None, None) == tao.ERR_SHAPE
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(R=0), None, None) == tao.ERR_SHAPE
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(H=2, R=5, ph=0), None, None) == tao.ERR_SHAPE   # filter > input
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(H=2 ** 28), None, None) == tao.ERR_SHAPE
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(B=2 ** 20, H=2 ** 10, W=2 ** 10), None, None) == tao.ERR_SHAPE  # rows >= 2^31
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(C=2 ** 22, R=2, S=2, ph=0, pw=0), None, None) == tao.ERR_K_RANGE
    assert L.tao_bound_conv2d(nul, p, nul, p, *cargs(), None, None) == tao.ERR_NULL
    assert L.tao_bound_conv2d(p, nul, nul, p, *cargs(), None, None) == tao.ERR_NULL
    assert L.tao_bound_conv2d(p, p, nul, odd, *cargs(), None, None) == tao.ERR_ALIGN
    assert L.tao_bound_conv2d(nul, nul, nul, nul, *cargs(B=0), None, None) == tao.OK
    assert L.tao_bound_conv2d(nul, nul, nul, nul, *cargs(Co=0), None, None) == tao.OK
    assert L.tao_bound_conv2d(p, p, nul, p, *cargs(), ctypes.byref(bad), None) == tao.ERR_MODEL
    # check
    need = L.tao_check_workspace_bytes(1000)
    assert need > 0
    ws = ctypes.c_void_p(0x10000)
    # softmax bound checked in one pass: (rows, cols, ld, alpha, eps_rel, model, out, ws, ws_bytes)
    assert L.tao_bound_check_softmax(p, p, p, 4, 8, 4, 1.0, 0.0, None, p, ws, need, None) == tao.ERR_SHAPE      # ld < cols
    assert L.tao_bound_check_softmax(p, p, nul, 4, 8, 8, 1.0, 0.0, None, p, ws, need, None) == tao.ERR_NULL
    assert L.tao_bound_check_softmax(p, p, p, 4, 8, 8, 1.0, 0.0, None, nul, ws, need, None) == tao.ERR_NULL
    assert L.tao_bound_check_softmax(p, p, p, 4, 8, 8, 1.0, 0.0, None, p, ws, need - 1, None) == tao.ERR_WORKSPACE
    assert L.tao_bound_check_softmax(p, odd, p, 4, 8, 8, 1.0, 0.0, None, p, ws, need, None) == tao.ERR_ALIGN
    assert L.tao_bound_check_softmax(p, p, p, 4, 2 ** 24 + 2, 2 ** 24 + 2, 1.0, 0.0, None, p, ws, need, None) == tao.ERR_K_RANGE
    assert L.tao_check_and_profile(p, p, p, 10, 1.0, 0.0, nul, ws, need, None) == tao.ERR_NULL
    assert L.tao_check_and_profile(p, p, p, 10, 1.0, 0.0, p, nul, need, None) == tao.ERR_WORKSPACE
    assert L.tao_check_and_profile(p, p, p, 10, 1.0, 0.0, p, ws, need - 1, None) == tao.ERR_WORKSPACE
    assert L.tao_check_and_profile(p, p, p, 10, 1.0, 0.0, p, ctypes.c_void_p(0x10010), need, None) == tao.ERR_WORKSPACE
    assert L.tao_check_and_profile(p, p, p, -1, 1.0, 0.0, p, ws, need, None) == tao.ERR_SHAPE
    assert L.tao_check_and_profile(p, p, p, 10, 1.0, -1e-9, p, ws, need, None) == tao.ERR_SHAPE      # negative eps_rel
    assert L.tao_check_and_profile(p, p, p, 10, 1.0, float("nan"), p, ws, need, None) == tao.ERR_SHAPE
    assert L.tao_check_and_profile(nul, p, p, 10, 1.0, 0.0, p, ws, need, None) == tao.ERR_NULL
    assert L.tao_check_and_profile(odd, p, p, 10, 1.0, 0.0, p, ws, need, None) == tao.ERR_ALIGN
    # error profiles
    need = L.tao_profile_workspace_bytes(1000)
    assert need > 0
    assert L.tao_profile_errors(p, p, 10, 0.0, nul, nul, nul, ws, need, None) == tao.ERR_NULL
    assert L.tao_profile_errors(p, p, 10, 0.0, nul, nul, p, nul, need, None) == tao.ERR_WORKSPACE
    assert L.tao_profile_errors(p, p, 10, 0.0, nul, nul, p, ws, need - 1, None) == tao.ERR_WORKSPACE
    assert L.tao_profile_errors(p, p, 10, 0.0, p, nul, p, ws, need, None) == tao.ERR_NULL      # one table only
    assert L.tao_profile_errors(p, nul, 10, 0.0, nul, nul, p, ws, need, None) == tao.ERR_NULL
    assert L.tao_profile_errors(p, p, -1, 0.0, nul, nul, p, ws, need, None) == tao.ERR_SHAPE
    assert L.tao_profile_errors(p, p, 10, -1.0, nul, nul, p, ws, need, None) == tao.ERR_SHAPE
    assert L.tao_profile_errors(odd, p, 10, 0.0, nul, nul, p, ws, need, None) == tao.ERR_ALIGN
    # calibration
    assert L.tao_calibrate_thresholds(p, 0, 3.0, nul, nul, p, p, None) == tao.ERR_SHAPE
    assert L.tao_calibrate_thresholds(p, 2, -1.0, nul, nul, p, p, None) == tao.ERR_SHAPE
    assert L.tao_calibrate_thresholds(nul, 2, 3.0, nul, nul, p, p, None) == tao.ERR_NULL
    assert L.tao_calibrate_thresholds(p, 2, 3.0, nul, nul, nul, p, None) == tao.ERR_NULL
    assert L.tao_calibrate_thresholds(odd, 2, 3.0, nul, nul, p, p, None) == tao.ERR_ALIGN
    # projections
    assert L.tao_project_clip(p, p, 1.0, p, -1, None) == tao.ERR_SHAPE
    assert L.tao_project_clip(p, p, -1.0, p, 10, None) == tao.ERR_SHAPE
    assert L.tao_project_clip(p, p, float("nan"), p, 10, None) == tao.ERR_SHAPE
    assert L.tao_project_clip(p, nul, 1.0, p, 10, None) == tao.ERR_NULL
    assert L.tao_project_clip(odd, p, 1.0, p, 10, None) == tao.ERR_ALIGN
    assert L.tao_project_clip(nul, nul, 1.0, nul, 0, None) == tao.OK
    need = L.tao_project_workspace_bytes(100000)
    assert 16 * 100000 <= need <= 16 * 100000 + (1 << 16)
    assert L.tao_project_workspace_bytes(0) == 0 and L.tao_project_workspace_bytes(1 << 31) == 0
    assert L.tao_project_workspace_bytes((1 << 31) - 1) > 16 * ((1 << 31) - 1)
    assert L.tao_project_empirical(p, p, 1.0, p, -1, ws, need, None) == tao.ERR_SHAPE
    assert L.tao_project_empirical(p, p, 1.0, p, 1 << 31, ws, 1 << 40, None) == tao.ERR_SHAPE
    assert L.tao_project_empirical(p, p, float("inf"), p, 100000, ws, need, None) == tao.ERR_SHAPE
    assert L.tao_project_empirical(p, nul, 1.0, p, 100000, ws, need, None) == tao.ERR_NULL
    assert L.tao_project_empirical(odd, p, 1.0, p, 100000, ws, need, None) == tao.ERR_ALIGN
    assert L.tao_project_empirical(p, p, 1.0, p, 100000, nul, need, None) == tao.ERR_WORKSPACE
    assert L.tao_project_empirical(p, p, 1.0, p, 100000, ws, need - 1, None) == tao.ERR_WORKSPACE
    assert L.tao_project_empirical(p, p, 1.0, p, 100000, ctypes.c_void_p(0x10010), need, None) == tao.ERR_WORKSPACE
    assert L.tao_project_empirical(nul, nul, 1.0, nul, 0, nul, 0, None) == tao.OK
    for code in range(0, -9, -1):
        assert L.tao_status_string(code)
    L.tao_selftest_workspace_bytes.restype = ctypes.c_size_t
    rep = ctypes.c_uint(0)
    assert L.tao_selftest_matrix_core(None, big, 8192, None) == tao.ERR_NULL
    assert L.tao_selftest_matrix_core(ctypes.byref(rep), nul, 8192, None) == tao.ERR_WORKSPACE     # scratch comes from the caller
    assert L.tao_selftest_matrix_core(ctypes.byref(rep), big, 100, None) == tao.ERR_WORKSPACE
    assert L.tao_selftest_matrix_core_bf16(None, 0, big, 1 << 20, None) == tao.ERR_NULL
    assert L.tao_selftest_matrix_core_bf16(ctypes.byref(rep), 0, nul, 1 << 20, None) == tao.ERR_WORKSPACE
    assert L.tao_selftest_matrix_core_bf16(ctypes.byref(rep), 280000, big, L.tao_selftest_workspace_bytes(280000) - 1, None) == tao.ERR_WORKSPACE
    assert L.tao_selftest_matrix_core_bf16(ctypes.byref(rep), -1, big, 1 << 20, None) == tao.ERR_SHAPE
    assert L.tao_selftest_workspace_bytes(0) == 3072 * 72 + 256 and L.tao_selftest_workspace_bytes(280000) == 280000 * 72 + 256


def test_binding_refuses_to_run_without_a_gpu(tao):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        tao.tao_bound_softmax(torch.zeros(2, 2), torch.zeros(2, 2))


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
