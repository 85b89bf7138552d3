"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element, on the benchmark configurations at sizes the oracle finishes in seconds, plus
edge cases.  Bounds: oracle <= gpu <= oracle (1 + 1e-6).  Check/profile: bit-exact."""
import numpy as np
import pytest
import torch

import tao_inputs
from opmap import assert_bound_parity, assert_profile_equal, gpu_tau, oracle_tau

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tao():
    import paper_2510_16028_amd as t
    t.lib()
    assert torch.cuda.is_available()
    return t


def _np(t):
    return t.detach().cpu().numpy()


def _run_ops(tao, oracle_mod, ops, expect_zero_violations=True):
    for op in ops:
        print("op", op.name, op.kind, tuple(op.y_ref.shape), flush=True)
        t_or = oracle_tau(oracle_mod, op)
        t_gpu = gpu_tau(tao, op)
        torch.cuda.synchronize()
        worst = assert_bound_parity(_np(t_gpu), t_or, op.name)
        print("   max tau_gpu/tau_oracle - 1 = %.3e" % worst, flush=True)
        # check + profile on identical inputs (the oracle's tau on both sides): bit-exact
        tau_dev = torch.from_numpy(np.ascontiguousarray(t_or)).cuda()
        pg = tao.tao_check_and_profile(op.claimed.cuda().contiguous(), op.y_ref.cuda().contiguous(), tau_dev)
        po = oracle_mod.check_and_profile(_np(op.claimed), _np(op.y_ref), t_or)
        assert_profile_equal(pg, po, op.name)
        if expect_zero_violations:
            assert pg["violations"] == 0 and pg["accept"] == 1, op.name
            # and the GPU's own bound accepts the honest claim as well
            pe = tao.tao_check_and_profile(op.claimed.cuda().contiguous(), op.y_ref.cuda().contiguous(),
                                           t_gpu.contiguous())
            assert pe["violations"] == 0, op.name


def test_matrix_core_selftest(tao):
    rep = tao.tao_selftest_matrix_core()
    print("matrix-core self test report:", rep, flush=True)
    assert rep & 1, "accumulation is not round-to-nearest-even"
    assert rep & 2, "subnormal products or operands are flushed"
    assert rep & 4, "6-step chain exceeds gamma_6"


def test_bf16_matrix_core_selftest(tao):
    rep = tao.tao_selftest_matrix_core_bf16()
    print("bf16 matrix-core self test report:", rep, flush=True)
    assert rep & 1, "v_mfma_f32_32x32x16_bf16 does not follow the model the split bound's inflation rests on"
    assert rep & 2, "a zero-accumulator instruction left [S(1-10u), S(1+2u)]"
    assert rep & 4, "a result in the subnormal range is more than two steps of 2^-149 from the exact sum"
    # the larger run on request: 280 000 cases of the same generator
    assert tao.tao_selftest_matrix_core_bf16(cases=280000) == 7
    assert tao.tao_linear_split_preferred(2048, 4096, 4096) and not tao.tao_linear_split_preferred(2048, 128, 2048, 8)
    # one column tile pays when A can be split while it is loaded (enough tiles, a long reduction of whole groups)
    assert tao.tao_linear_split_preferred(8192, 128, 2048, 8) and not tao.tao_linear_split_preferred(8192, 128, 2040, 8)
    # few tiles: preferred where the reduction, cut into parts, fills the chip
    assert tao.tao_linear_split_preferred(512, 768, 768) and not tao.tao_linear_split_preferred(128, 768, 768)


def test_config1_linear_and_softmax(tao, oracle_mod):
    ops = tao_inputs.config1("cpu")
    _run_ops(tao, oracle_mod, ops)
    # closed form of the workload: +-{0..3} ulp noise => max relative error <= 3 * 2^-23
    p = tao.tao_check_and_profile(ops[0].claimed.cuda(), ops[0].y_ref.cuda(),
                                  gpu_tau(tao, ops[0]), eps_rel=0.0)
    assert p["violations"] == 0 and 0 < p["max_rel"] <= np.float32(3 * 2.0 ** -23)


def test_config2_bert_block_scaled(tao, oracle_mod):
    _run_ops(tao, oracle_mod, tao_inputs.config2("cpu", scale=4))


def test_config3_qwen_layer_scaled(tao, oracle_mod):
    _run_ops(tao, oracle_mod, tao_inputs.config3("cpu", scale=16))


def test_config4_conv_stage_scaled(tao, oracle_mod):
    _run_ops(tao, oracle_mod, tao_inputs.config4("cpu", scale=32))


def test_config5_stress_scaled(tao, oracle_mod):
    g, A, W = tao_inputs.config5_operands("cpu", size=384)
    ref = A @ W.t()
    t_or = oracle_mod.bound_linear(_np(A), _np(W))
    t_gpu = tao.tao_bound_linear(A.cuda(), W.cuda())
    assert_bound_parity(_np(t_gpu), t_or, "c5 linear")
    claimed, cls = tao_inputs.config5_claimed(g, ref, torch.from_numpy(t_or))
    po = oracle_mod.check_and_profile(_np(claimed), _np(ref), t_or)
    assert po["violations"] == int((cls == 2).sum())            # the 1.01x class, known from the seed
    pg = tao.tao_check_and_profile(claimed.cuda(), ref.cuda(), torch.from_numpy(t_or).cuda())
    assert_profile_equal(pg, po, "c5 check")
    # the GPU's own bound gives the same violation counts: 1 % margins >> 1e-6 tolerance
    pe = tao.tao_check_and_profile(claimed.cuda(), ref.cuda(), t_gpu)
    assert pe["violations"] == po["violations"]


@pytest.mark.parametrize("M,N,K,bias,trans_w,batch", [
    (1, 1, 1, False, False, 1), (1, 5, 7, True, False, 1), (129, 257, 49, True, False, 1),
    (130, 64, 601, False, True, 1), (33, 200, 48, True, True, 3), (256, 128, 96, False, False, 2),
    (5, 3, 0, True, False, 1), (70, 130, 13, False, False, 1)])
def test_linear_shapes(tao, oracle_mod, M, N, K, bias, trans_w, batch):
    g = torch.Generator().manual_seed(M * 1000 + N * 10 + K)
    A = torch.randn((batch, M, K), generator=g)
    W = torch.randn((batch, K, N) if trans_w else (batch, N, K), generator=g)
    b = torch.randn((N,), generator=g) if bias else None
    if batch == 1:
        A, W = A[0], W[0]
    t_or = oracle_mod.bound_linear(_np(A), _np(W), None if b is None else _np(b), trans_w=trans_w)
    t_gpu = tao.tao_bound_linear(A.cuda(), W.cuda(), None if b is None else b.cuda(), trans_w=trans_w)
    assert_bound_parity(_np(t_gpu), t_or, "linear %s" % ((M, N, K, bias, trans_w, batch),))


@pytest.mark.parametrize("M,N,K,bias,trans_w,batch", [
    (2048, 2560, 64, True, False, 1),      # 320 tiles of 128 rows: persistent walk, several groups per tile
    (2048, 2560, 96, False, True, 1),      # same with W stored K x N
    (3840, 1280, 160, True, True, 1),      # 300 / 600 tiles: 64-row tiles make fewer, cheaper rounds; persistent
    (512, 640, 32, False, False, 5),       # batched, one k-slab per tile: the shortest pipeline
    (384, 384, 224, True, False, 3),       # batched 64-row tiles, odd number of groups
    (1920, 1280, 64, False, True, 2),      # batched, 64-row tiles, persistent across batch entries
    (1024, 1024, 1056, False, False, 1),   # just past the persistent limit: one tile per workgroup
])
def test_linear_aligned_tile_walks(tao, oracle_mod, M, N, K, bias, trans_w, batch):
    """Aligned shapes take the buffer-load pipeline; with more tiles than compute units and a
    short K loop each workgroup walks several tiles. Every element against the oracle."""
    g = torch.Generator().manual_seed(M + 7 * N + 13 * K + batch)
    A = torch.randn((batch, M, K), generator=g)
    W = torch.randn((batch, K, N) if trans_w else (batch, N, K), generator=g)
    b = torch.randn((N,), generator=g) if bias else None
    if batch == 1:
        A, W = A[0], W[0]
    t_or = oracle_mod.bound_linear(_np(A), _np(W), None if b is None else _np(b), trans_w=trans_w)
    t_gpu = tao.tao_bound_linear(A.cuda(), W.cuda(), None if b is None else b.cuda(), trans_w=trans_w)
    assert_bound_parity(_np(t_gpu), t_or, "linear %s" % ((M, N, K, bias, trans_w, batch),))
    fast = tao.tao_bound_linear(A.cuda(), W.cuda(), None if b is None else b.cuda(), trans_w=trans_w,
                                model=tao.FpModel(flags=tao.FLAG_FAST_ACCUM))
    assert_bound_parity(_np(fast), t_or, "fast", rel_tol=2.5 * max(K, 1) * 2.0 ** -24)


@pytest.mark.parametrize("B,H,W,C,Cout,R,S,stride,pad,dil,bias", [
    (2, 16, 16, 32, 128, 3, 3, (1, 1), (1, 1), (1, 1), True),     # gather path, 512 patch rows, padding on all sides
    (1, 32, 24, 64, 256, 3, 3, (1, 1), (1, 1), (1, 1), False),    # gather path, two column tiles, two slabs per tap
    (2, 17, 19, 32, 128, 3, 2, (2, 1), (0, 1), (1, 2), True),     # stride, dilation, ragged row tile (gather + edge tiles)
    (1, 31, 33, 96, 128, 1, 1, (2, 2), (0, 0), (1, 1), False),    # 1 x 1 strided (a projection shortcut)
    (3, 9, 11, 3, 5, 7, 7, (2, 2), (3, 3), (1, 1), True),         # stem-like: 3 channels, element path
    (1, 8, 8, 40, 130, 3, 3, (1, 1), (2, 2), (2, 2), False),      # channels not a multiple of 32, ragged columns
    (2, 6, 5, 32, 64, 5, 5, (1, 1), (2, 2), (1, 1), True),        # filter as large as the input
    (1, 4, 4, 32, 128, 3, 3, (1, 1), (3, 3), (1, 1), False),      # outputs whose taps all fall into the padding
    (1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0), (1, 1), True),
    (8, 56, 56, 64, 128, 3, 3, (1, 1), (1, 1), (1, 1), True),     # 196 tiles of 128 rows: the large-tile gather kernel
])
def test_conv2d_shapes(tao, oracle_mod, B, H, W, C, Cout, R, S, stride, pad, dil, bias):
    """The implicit-patch-matrix convolution bound against the oracle's direct triple loop,
    every output element; both accumulation modes."""
    g = torch.Generator().manual_seed(B + 3 * H + 5 * W + 7 * C + 11 * Cout + 13 * R)
    x = torch.randn((B, H, W, C), generator=g)
    w = torch.randn((Cout, R, S, C), generator=g) * 0.1
    b = torch.randn((Cout,), generator=g) if bias else None
    t_or = oracle_mod.bound_conv2d(_np(x), _np(w), None if b is None else _np(b), stride, pad, dil)
    t_gpu = tao.tao_bound_conv2d(x.cuda(), w.cuda(), None if b is None else b.cuda(), stride, pad, dil)
    assert tuple(t_gpu.shape) == t_or.shape
    assert_bound_parity(_np(t_gpu), t_or, "conv %s" % ((B, H, W, C, Cout, R, S, stride, pad, dil),))
    fast = tao.tao_bound_conv2d(x.cuda(), w.cuda(), None if b is None else b.cuda(), stride, pad, dil,
                                model=tao.FpModel(flags=tao.FLAG_FAST_ACCUM))
    assert_bound_parity(_np(fast), t_or, "conv fast", rel_tol=2.5 * R * S * C * 2.0 ** -24)


def test_conv2d_accepts_a_real_convolution(tao, oracle_mod):
    """A binary32 convolution computed by another algorithm (torch on the CPU, NCHW) against the
    binary64 reference: every error within the GPU's bound, and the bound identical whether the
    operand is a channels-last view of an NCHW tensor or a plain NHWC tensor."""
    g = torch.Generator().manual_seed(9)
    x = torch.randn((2, 64, 14, 14), generator=g)
    w = torch.randn((128, 64, 3, 3), generator=g) * 0.05
    y32 = torch.nn.functional.conv2d(x, w, padding=1)
    y64 = torch.nn.functional.conv2d(x.double(), w.double(), padding=1)
    xl = x.cuda().contiguous(memory_format=torch.channels_last).permute(0, 2, 3, 1)
    wl = w.cuda().contiguous(memory_format=torch.channels_last).permute(0, 2, 3, 1)
    assert xl.is_contiguous() and wl.is_contiguous()
    tau = tao.tao_bound_conv2d(xl, wl, None, 1, 1, 1)
    err = (y32.double() - y64).abs().permute(0, 2, 3, 1)
    assert bool((err <= tau.cpu().double()).all())
    t_or = oracle_mod.bound_conv2d(_np(xl), _np(wl), None, (1, 1), (1, 1), (1, 1))
    assert_bound_parity(_np(tau), t_or, "conv nchw view")


@pytest.mark.parametrize("M,N,K,bias,trans_w,batch", [
    (1, 1, 1, False, False, 1), (1, 5, 7, True, False, 1), (129, 257, 49, True, False, 1),
    (130, 64, 601, False, True, 1), (33, 200, 48, True, True, 3), (256, 128, 96, False, False, 2),
    (5, 3, 0, True, False, 1), (70, 130, 13, False, False, 1), (512, 384, 2048, True, False, 1),
    (2048, 256, 64, False, True, 2), (384, 384, 1088, True, False, 3),
    # fewer tiles than compute units and a long reduction: cut into parts (the first, K = 2048, and the
    # one before are too), parts of unequal length, the shape of configuration 3's k/v projections
    (200, 300, 1500, True, False, 1), (2048, 1024, 4096, False, False, 1),
    # short reductions with many tiles per compute unit: a workgroup walks several tiles (ragged edges,
    # so many of its slots hold no tile; the second has the shortest reduction that walks)
    (2100, 1500, 100, True, False, 6), (1100, 2300, 40, False, True, 4),
    # as many tiles, but a single group per tile: too short to walk, one workgroup per tile
    (2100, 1500, 20, True, False, 6)])
def test_linear_split_shapes(tao, oracle_mod, M, N, K, bias, trans_w, batch):
    """The BF16-split path against the oracle, every element (same tolerance as the FP32 path)."""
    g = torch.Generator().manual_seed(M * 1000 + N * 10 + K + 5)
    A = torch.randn((batch, M, K), generator=g)
    W = torch.randn((batch, K, N) if trans_w else (batch, N, K), generator=g)
    b = torch.randn((N,), generator=g) if bias else None
    if batch == 1:
        A, W = A[0], W[0]
    t_or = oracle_mod.bound_linear(_np(A), _np(W), None if b is None else _np(b), trans_w=trans_w)
    t_gpu = tao.tao_bound_linear_split(A.cuda(), W.cuda(), None if b is None else b.cuda(), trans_w=trans_w)
    worst = assert_bound_parity(_np(t_gpu), t_or, "split linear %s" % ((M, N, K, bias, trans_w, batch),))
    print("max tau_gpu/tau_oracle - 1 = %.3e" % worst, flush=True)


def test_linear_split_value_ranges_and_shared_w(tao, oracle_mod):
    """Wide dynamic range inside the reduction (the truncation steps of the instruction bite
    there), heavy tails, exact powers of two, a W shared across the batch, infinities."""
    g = torch.Generator().manual_seed(808)
    M, N, K = 96, 160, 320
    expo = torch.randint(-20, 21, (M, K), generator=g).float()
    A = torch.randn((M, K), generator=g) * 2.0 ** expo
    W = torch.randn((N, K), generator=g) * 2.0 ** torch.randint(-12, 13, (N, K), generator=g).float()
    for a, w, what in ((A, W, "wide exponents"), (2.0 ** expo, torch.ones(N, K), "powers of two"),
                       (A * 1e-25, W * 1e-8, "small magnitudes"), (A * 1e15, W * 1e10, "large magnitudes")):
        t_or = oracle_mod.bound_linear(_np(a), _np(w))
        assert_bound_parity(_np(tao.tao_bound_linear_split(a.cuda(), w.cuda())), t_or, what)
    A3 = torch.randn((3, M, K), generator=g)
    t_or = oracle_mod.bound_linear(_np(A3), _np(W[None]))
    t_gpu = tao.tao_bound_linear_split(A3.cuda(), W.cuda()[None].expand(3, N, K))
    assert_bound_parity(_np(t_gpu), t_or, "shared W")
    # an infinite operand: the oracle's row is +inf; a piece of the other operand that is exactly
    # zero turns inf into NaN on the matrix cores, so the row is +inf or NaN (never finite)
    Ai = A.clone(); Ai[2, 5] = float("inf")
    t_or = oracle_mod.bound_linear(_np(Ai), _np(W))
    t_gpu = _np(tao.tao_bound_linear_split(Ai.cuda(), W.cuda()))
    assert np.all(np.isinf(t_or[2])) and not np.any(np.isfinite(t_gpu[2]))
    keep = np.arange(M) != 2
    assert_bound_parity(t_gpu[keep], t_or[keep], "rows beside an infinite operand")


def test_linear_random_shapes_and_strides(tao, oracle_mod):
    """Forty seeded shapes around the tile and slab sizes, with padded row strides, batches,
    either W layout and optional bias: every element against the oracle."""
    rng = np.random.Generator(np.random.Philox(2024))
    edges = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 255, 256, 257]
    for case in range(40):
        M = int(rng.choice(edges)) if rng.random() < 0.6 else int(rng.integers(1, 300))
        N = int(rng.choice(edges)) if rng.random() < 0.6 else int(rng.integers(1, 300))
        K = int(rng.choice(edges + [0, 4, 96, 160])) if rng.random() < 0.6 else int(rng.integers(1, 300))
        batch = int(rng.integers(1, 4))
        trans_w = bool(rng.integers(0, 2)); bias = bool(rng.integers(0, 2))
        pad_a, pad_w = int(rng.choice([0, 0, 1, 4, 7])), int(rng.choice([0, 0, 3, 4, 12]))
        g = torch.Generator().manual_seed(1000 + case)
        Afull = torch.randn((batch, M, K + pad_a), generator=g)
        wshape = (batch, K, N + pad_w) if trans_w else (batch, N, K + pad_w)
        Wfull = torch.randn(wshape, generator=g)
        b = torch.randn((N,), generator=g) if bias else None
        A = Afull[:, :, :K]; W = Wfull[:, :, :N] if trans_w else Wfull[:, :, :K]
        what = "case %d: M=%d N=%d K=%d batch=%d trans_w=%s bias=%s pads=(%d,%d)" % (case, M, N, K, batch, trans_w, bias, pad_a, pad_w)
        print(what, flush=True)
        t_or = oracle_mod.bound_linear(_np(A.contiguous()), _np(W.contiguous()), None if b is None else _np(b), trans_w=trans_w)
        Ag = Afull.cuda()[:, :, :K]; Wg = Wfull.cuda()[:, :, :N] if trans_w else Wfull.cuda()[:, :, :K]
        bg = None if b is None else b.cuda()
        assert_bound_parity(_np(tao.tao_bound_linear(Ag, Wg, bg, trans_w=trans_w)), t_or, what)
        assert_bound_parity(_np(tao.tao_bound_linear_split(Ag, Wg, bg, trans_w=trans_w)), t_or, what + " (bf16 split)")


def test_conv2d_random_geometries(tao, oracle_mod):
    """Thirty seeded convolution geometries (strides, paddings, dilations, channel counts on both
    sides of the 32-channel gather path) against the oracle's direct loop."""
    rng = np.random.Generator(np.random.Philox(2025))
    for case in range(30):
        C = int(rng.choice([1, 3, 8, 32, 32, 64, 96, 40]))
        Cout = int(rng.choice([1, 5, 64, 128, 128, 130, 256]))
        R, S = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        dh, dw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        H = int(rng.integers(max(1, dh * (R - 1) + 1 - 2 * ph), 20)); W = int(rng.integers(max(1, dw * (S - 1) + 1 - 2 * pw), 20))
        B = int(rng.integers(1, 4))
        what = "case %d: B=%d H=%d W=%d C=%d Cout=%d R=%d S=%d stride=(%d,%d) pad=(%d,%d) dil=(%d,%d)" % (
            case, B, H, W, C, Cout, R, S, sh, sw, ph, pw, dh, dw)
        print(what, flush=True)
        g = torch.Generator().manual_seed(3000 + case)
        x = torch.randn((B, H, W, C), generator=g); w = torch.randn((Cout, R, S, C), generator=g)
        b = torch.randn((Cout,), generator=g) if case % 2 else None
        t_or = oracle_mod.bound_conv2d(_np(x), _np(w), None if b is None else _np(b), (sh, sw), (ph, pw), (dh, dw))
        t_gpu = tao.tao_bound_conv2d(x.cuda(), w.cuda(), None if b is None else b.cuda(), (sh, sw), (ph, pw), (dh, dw))
        assert_bound_parity(_np(t_gpu), t_or, what)


@pytest.mark.parametrize("B,H,W,C,Cout,R,S,stride,pad,dil", [
    (20, 40, 40, 32, 128, 3, 3, (1, 1), (1, 1), (1, 1)),      # 250 tiles of one column tile
    (33, 33, 35, 64, 200, 3, 3, (1, 1), (1, 1), (1, 1)),      # ragged rows and columns, two column tiles
    (40, 29, 31, 32, 130, 5, 3, (1, 2), (3, 0), (2, 1)),      # strides, asymmetric padding, dilation: taps in the padding
    (36, 30, 30, 96, 64, 1, 1, (1, 1), (0, 0), (1, 1)),       # 1 x 1: a plain product with three groups
])
def test_conv2d_bound_on_the_bf16_matrix_cores(tao, oracle_mod, B, H, W, C, Cout, R, S, stride, pad, dil):
    """tao_bound_conv2d_split / tao_bound_check_conv2d: parity with the oracle's direct loop (on a few
    images), the bits of the BF16-split product on the explicit patch matrix, and the checked variant's
    profile against the two separate calls."""
    assert tao.tao_conv2d_split_supported((B, H, W, C), (Cout, R, S, C), stride, pad, dil)
    g = torch.Generator(device="cuda").manual_seed(B * 31 + C + Cout)
    x = torch.randn((B, H, W, C), generator=g, device="cuda").abs()
    w = torch.randn((Cout, R, S, C), generator=g, device="cuda") * 0.05
    b = torch.randn((Cout,), generator=g, device="cuda")
    tau = tao.tao_bound_conv2d_split(x, w, b, stride, pad, dil)
    for img in (0, B - 1):
        t_or = oracle_mod.bound_conv2d(_np(x[img:img + 1]), _np(w), _np(b), stride, pad, dil)
        assert_bound_parity(_np(tau[img:img + 1]), t_or, "conv on BF16 cores, image %d" % img)
    # the explicit patch matrix (columns ordered (r, s, c) like the filters) through the matrix entry point
    xp = torch.nn.functional.pad(x.permute(0, 3, 1, 2), (pad[1], pad[1], pad[0], pad[0]))
    cols = torch.nn.functional.unfold(xp, kernel_size=(R, S), dilation=dil, stride=stride)          # [B, C*R*S, L], (c, r, s) order
    L = cols.shape[-1]
    A = cols.reshape(B, C, R * S, L).permute(0, 3, 2, 1).reshape(B * L, R * S * C).contiguous()
    via_matrix = tao.tao_bound_linear_split(A, w.reshape(Cout, -1), b)
    assert torch.equal(via_matrix.view(torch.int32).reshape(-1), tau.view(torch.int32).reshape(-1))
    # checked on the spot
    ref = (A @ w.reshape(Cout, -1).t() + b).contiguous()
    claimed = tao_inputs.ulp_noise(g, ref, max_ulps=2)
    claimed.view(-1)[5] += 1.0
    tau2 = torch.empty_like(tau)
    one = tao.tao_bound_check_conv2d(x, w, b, ref, claimed, stride, pad, dil, tau_out=tau2)
    assert torch.equal(tau2.view(torch.int32), tau.view(torch.int32))
    assert_profile_equal(one, tao.tao_check_and_profile(claimed.reshape(-1), ref.reshape(-1), tau.reshape(-1)), "conv checked on the spot")
    assert one["violations"] >= 1
    # shapes it does not serve are refused, not mangled
    with pytest.raises(tao.TaoError) as ei:
        tao.tao_bound_conv2d_split(x[:, :, :, :24].contiguous(), w[:, :, :, :24].contiguous(), b, stride, pad, dil)
    assert ei.value.status == tao.ERR_SHAPE


def test_linear_unaligned_views_and_modes(tao, oracle_mod):
    g = torch.Generator().manual_seed(77)
    Abig = torch.randn((150, 203), generator=g).cuda()
    Wbig = torch.randn((90, 203), generator=g).cuda()
    A = Abig[:, 1:200]            # row stride 203, base misaligned by 4 bytes
    W = Wbig[:, 3:202]
    t_or = oracle_mod.bound_linear(_np(A), _np(W))
    assert_bound_parity(_np(tao.tao_bound_linear(A, W)), t_or, "strided views")
    # probabilistic constant (Sec. 3.1, lambda = 4)
    mo, mg = oracle_mod.Model(mode=1), tao.FpModel(mode=1)
    assert_bound_parity(_np(tao.tao_bound_linear(A, W, model=mg)),
                        oracle_mod.bound_linear(_np(A), _np(W), model=mo), "probabilistic")
    # underflow term
    mo, mg = oracle_mod.Model(flags=1), tao.FpModel(flags=tao.FLAG_UNDERFLOW_TERMS)
    tiny = (A * 1e-30, W * 1e-12)
    # (with the flag the bound carries absolute terms of the order of the subnormal step itself, on both
    # sides: the flag's contract is the reference's value or the next binary32 value above it)
    t_uf, t_uf_or = _np(tao.tao_bound_linear(tiny[0], tiny[1], model=mg)), oracle_mod.bound_linear(_np(tiny[0]), _np(tiny[1]), model=mo)
    assert np.all(t_uf >= t_uf_or) and np.all(t_uf <= np.nextafter(t_uf_or * np.float32(1 + 1e-6), np.float32(np.inf)))
    # single-chain accumulation: still never below the oracle, looser by at most ~2 K u
    fast = _np(tao.tao_bound_linear(A, W, model=tao.FpModel(flags=tao.FLAG_FAST_ACCUM)))
    K = A.shape[1]
    assert_bound_parity(fast, t_or, "fast accumulation", rel_tol=2.5 * K * 2.0 ** -24)


@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 2), (64, 128), (7, 257), (33, 512), (5, 1000),
                                       (9, 2048), (4, 4100), (3, 8192), (2, 9001)])
def test_softmax_shapes(tao, oracle_mod, rows, cols):
    g = torch.Generator().manual_seed(rows * 100003 + cols)
    x = torch.randn((rows, cols), generator=g) * 3
    if cols > 2:
        x[0, cols // 2:] = float("-inf")                   # partly masked row
    if rows > 2:
        x[1, :] = float("-inf")                            # fully masked row -> NaN
        x[2, 0] = float("nan")                             # poisoned row -> NaN
    y = tao_inputs.softmax_f32(x)
    y = torch.nan_to_num(y, nan=0.0)
    t_or = oracle_mod.bound_softmax(_np(x), _np(y))
    t_gpu = tao.tao_bound_softmax(x.cuda(), y.cuda())
    assert_bound_parity(_np(t_gpu), t_or, "softmax %dx%d" % (rows, cols))


def test_softmax_padded_rows_and_probabilistic(tao, oracle_mod):
    g = torch.Generator().manual_seed(5)
    big = torch.randn((20, 301), generator=g)
    x = big[:, :299]
    y = tao_inputs.softmax_f32(x.contiguous())
    ybig = torch.zeros_like(big); ybig[:, :299] = y
    t_gpu = tao.tao_bound_softmax(big.cuda()[:, :299], ybig.cuda()[:, :299])
    assert_bound_parity(_np(t_gpu), oracle_mod.bound_softmax(_np(x.contiguous()), _np(y)), "padded softmax")
    t_p = tao.tao_bound_softmax(x.contiguous().cuda(), y.cuda(), model=tao.FpModel(mode=1, c_exp=3.0))
    assert_bound_parity(_np(t_p), oracle_mod.bound_softmax(_np(x.contiguous()), _np(y),
                                                          model=oracle_mod.Model(mode=1, c_exp=3.0)), "prob softmax")


@pytest.mark.parametrize("kind", ["layernorm", "rmsnorm", "bn_affine", "sum", "mean"])
@pytest.mark.parametrize("rows,cols", [(1, 1), (5, 3), (16, 256), (7, 768), (3, 1030), (4, 4096), (2, 8200)])
def test_norm_shapes(tao, oracle_mod, kind, rows, cols):
    g = torch.Generator().manual_seed(rows * 7919 + cols)
    x = torch.randn((rows, cols), generator=g) * 2 + 0.5
    gam = 1 + 0.1 * torch.randn((cols,), generator=g)
    bet = 0.1 * torch.randn((cols,), generator=g)
    code = {"layernorm": 0, "rmsnorm": 1, "bn_affine": 2, "sum": 3, "mean": 4}[kind]
    eps = 1e-5
    if kind == "layernorm":
        y = tao_inputs.layernorm_f32(x, gam, bet, eps)
    elif kind == "rmsnorm":
        y = tao_inputs.rmsnorm_f32(x, gam, eps)
    elif kind == "bn_affine":
        y = x * gam + bet
    elif kind == "sum":
        y = None
    else:
        y = x.sum(-1) / cols
    t_or = oracle_mod.bound_norm(code, _np(x), y=None if y is None else _np(y), g=_np(gam), b=_np(bet), eps=eps)
    t_gpu = tao.tao_bound_norm(code, x.cuda(), None if y is None else y.cuda(), gam.cuda(), bet.cuda(), eps=eps)
    assert_bound_parity(_np(t_gpu), t_or, "%s %dx%d" % (kind, rows, cols))


@pytest.mark.parametrize("cols", [1 << 20, (1 << 22) + 3, 1 << 23])
def test_very_long_rows(tao, oracle_mod, cols):
    """One row of millions of columns: the reference adds the row sequentially with upward rounding
    (up to cols 2^-52 above the real sum) and the kernels add it as a tree in round-to-nearest, so the
    margin of the kernels' final upper rounding has to grow with the row length for the bound to
    stay at or above the reference's -- and the whole still has to fit the 1e-6 tolerance."""
    g = torch.Generator().manual_seed(cols)
    x = torch.randn((1, cols), generator=g) + 0.25
    gam = 1 + 0.1 * torch.randn((cols,), generator=g)
    bet = 0.1 * torch.randn((cols,), generator=g)
    xs = x * 3
    ys = tao_inputs.softmax_f32(xs)
    assert_bound_parity(_np(tao.tao_bound_softmax(xs.cuda(), ys.cuda())), oracle_mod.bound_softmax(_np(xs), _np(ys)),
                        "softmax 1x%d" % cols)
    for kind, code in (("sum", 3), ("mean", 4), ("rmsnorm", 1), ("layernorm", 0)):
        if kind == "sum":
            y = None
        elif kind == "mean":
            y = x.sum(-1) / cols
        elif kind == "rmsnorm":
            y = tao_inputs.rmsnorm_f32(x, gam, 1e-6)
        else:
            y = tao_inputs.layernorm_f32(x, gam, bet, 1e-6)
        if code in (0, 1) and cols > 5_590_000:
            # Gamma(n - 1) > 1/2: the variance's error bound has eaten the variance; refused
            with pytest.raises(tao.TaoError) as ei:
                tao.tao_bound_norm(code, x.cuda(), y.cuda(), gam.cuda(), bet.cuda(), eps=1e-6)
            assert ei.value.status == tao.ERR_K_RANGE
            continue
        t_or = oracle_mod.bound_norm(code, _np(x), y=None if y is None else _np(y), g=_np(gam), b=_np(bet), eps=1e-6)
        t_gpu = tao.tao_bound_norm(code, x.cuda(), None if y is None else y.cuda(), gam.cuda(), bet.cuda(), eps=1e-6)
        worst = assert_bound_parity(_np(t_gpu), t_or, "%s 1x%d" % (kind, cols))
        print("   %s 1x%d: max tau_gpu/tau_oracle - 1 = %.3e" % (kind, cols, worst), flush=True)


def test_bounds_in_the_subnormal_range(tao, oracle_mod):
    """Bounds that land among the binary32 subnormals (one step there is a large relative amount):
    the kernels round such values up exactly, so they agree with the reference to the stated
    tolerance without any absolute allowance."""
    g = torch.Generator().manual_seed(4242)
    # softmax rows with a wide spread: most outputs, and their bounds, are tiny or zero
    x = torch.randn((64, 300), generator=g) * 25
    y = tao_inputs.softmax_f32(x)
    t_or = oracle_mod.bound_softmax(_np(x), _np(y))
    assert ((t_or > 0) & (t_or < 2.0 ** -126)).sum() > 100
    assert_bound_parity(_np(tao.tao_bound_softmax(x.cuda(), y.cuda())), t_or, "softmax, subnormal bounds")
    # element-wise kinds and the row kernels on outputs scaled into the subnormal range
    ysm = (torch.randn((8, 1000), generator=g) * 1e-33).contiguous()
    xsm = torch.randn((8, 1000), generator=g)
    for kind in (0, 1, 2, 6, 17):
        t_or = oracle_mod.bound_act(kind, _np(xsm * 1e-32), _np(ysm))
        assert_bound_parity(_np(tao.tao_bound_act(kind, (xsm * 1e-32).cuda(), ysm.cuda())), t_or, "act %d, subnormal bounds" % kind)
    gam = (torch.randn((1000,), generator=g) * 1e-34).contiguous()
    for code in (0, 1, 2):
        t_or = oracle_mod.bound_norm(code, _np(xsm), y=_np(ysm), g=_np(gam), b=None, eps=1e-5)
        assert ((t_or > 0) & (t_or < 2.0 ** -126)).sum() > 100
        assert_bound_parity(_np(tao.tao_bound_norm(code, xsm.cuda(), ysm.cuda(), gam.cuda(), None, eps=1e-5)), t_or,
                            "norm %d, subnormal bounds" % code)
    cs = torch.cos(torch.arange(32 * 64, dtype=torch.float32).reshape(32, 64) * 0.01)
    sn = torch.sin(torch.arange(32 * 64, dtype=torch.float32).reshape(32, 64) * 0.01)
    xr = (torch.randn((32, 128), generator=g) * 1e-33).contiguous()
    assert_bound_parity(_np(tao.tao_bound_rope(xr.cuda(), cs.cuda(), sn.cuda(), inner=1)),
                        oracle_mod.bound_rope(_np(xr), _np(cs), _np(sn), inner=1), "rope, subnormal bounds")


def test_linear_tiny_operands_stay_above_the_reference(tao, oracle_mod):
    """Operands so small that products and partial sums fall into the binary32 subnormal range (or
    below it), with default flags: the matrix cores round such values absolutely, not relatively,
    so the bound carries an absolute term for its own evaluation and may exceed 1e-6 there -- but
    it never falls below the reference, which forms the products exactly in binary64."""
    g = torch.Generator().manual_seed(99)
    for sa, sw in ((1e-30, 1e-12), (1e-20, 1e-20), (1e-25, 1e-12), (1e-38, 1.0), (1e-19, 1e-19)):
        for M, N, K in ((70, 130, 200), (128, 128, 64), (33, 17, 1031)):
            A = torch.randn((M, K), generator=g) * sa
            W = torch.randn((N, K), generator=g) * sw
            t_or = oracle_mod.bound_linear(_np(A), _np(W))
            t_gpu = _np(tao.tao_bound_linear(A.cuda(), W.cuda()))
            assert np.all(t_gpu >= t_or), "FP32 path below the reference at scales %g x %g: %d elements" % (
                sa, sw, int((t_gpu < t_or).sum()))
            # the excess is the absolute term: Gamma(K) (1.25 K + 40) 2^-150, i.e. a few subnormal steps
            K_ = float(K)
            slack = (K_ * 2.0 ** -24 / (1 - K_ * 2.0 ** -24)) * (1.25 * K_ + 40) * 2.0 ** -150 * 1.01
            assert np.all(t_gpu <= t_or.astype(np.float64) * (1 + 1e-6) + slack + 2.0 ** -149)
            # the same operands through the BF16-split path (its absolute term: Gamma(K) (Kp + 32) 2^-149)
            t_split = _np(tao.tao_bound_linear_split(A.cuda(), W.cuda()))
            assert np.all(t_split >= t_or), "BF16 path below the reference at scales %g x %g: %d elements" % (
                sa, sw, int((t_split < t_or).sum()))
            Kp = float((K + 31) // 32 * 32)
            slack = (K_ * 2.0 ** -24 / (1 - K_ * 2.0 ** -24)) * (Kp + 32) * 2.0 ** -149 * 1.01
            if min(sa, sw) >= 1e-25:           # operands below 2^-110 round their third piece up: sound, looser
                assert np.all(t_split <= t_or.astype(np.float64) * (1 + 1e-6) + slack + 2.0 ** -149)
    # products that vanish altogether (every one below 2^-150): with the underflow terms the bound still
    # covers the reference, which adds K' 2^-149 to the exact sum
    mo, mg = oracle_mod.Model(flags=1), tao.FpModel(flags=tao.FLAG_UNDERFLOW_TERMS)
    A = torch.randn((70, 200), generator=g) * 1e-30
    W = torch.randn((130, 200), generator=g) * 1e-20
    t_or = oracle_mod.bound_linear(_np(A), _np(W), model=mo)
    for t_gpu in (_np(tao.tao_bound_linear(A.cuda(), W.cuda(), model=mg)), _np(tao.tao_bound_linear_split(A.cuda(), W.cuda(), model=mg))):
        assert np.all(t_gpu >= t_or) and np.all(t_gpu <= t_or + np.float32(2.0 ** -149))


@pytest.mark.parametrize("kind", ["layernorm", "rmsnorm", "bn_affine", "mean"])
@pytest.mark.parametrize("rows,cols", [(1, 1), (5, 3), (16, 256), (7, 768), (3, 1030), (4, 4096), (2, 8200), (3, 20000)])
def test_norm_bounds_without_the_reexecuted_output(tao, oracle_mod, kind, rows, cols):
    """y_ref = NULL: the fresh-rounding term at the template's own upper bound of |y|; against the
    oracle, with and without scale and shift, and never below the bound that is given y."""
    g = torch.Generator().manual_seed(rows * 977 + cols)
    x = torch.randn((rows, cols), generator=g) * 2 + 0.5
    gam = 1 + 0.1 * torch.randn((cols,), generator=g)
    bet = 0.5 * torch.randn((cols,), generator=g)
    code = {"layernorm": 0, "rmsnorm": 1, "bn_affine": 2, "mean": 4}[kind]
    eps = 1e-5
    variants = [(gam, bet), (gam, None)] + ([] if kind == "bn_affine" else [(None, None)])
    for gg, bb in variants:
        t_or = oracle_mod.bound_norm(code, _np(x), y=None, g=None if gg is None else _np(gg), b=None if bb is None else _np(bb), eps=eps)
        t_gpu = tao.tao_bound_norm(code, x.cuda(), None, None if gg is None else gg.cuda(), None if bb is None else bb.cuda(), eps=eps)
        assert_bound_parity(_np(t_gpu), t_or, "%s %dx%d without y" % (kind, rows, cols))
    # the bound that knows an actual output is never larger
    if kind == "layernorm":
        y = tao_inputs.layernorm_f32(x, gam, bet, eps)
    elif kind == "rmsnorm":
        y = tao_inputs.rmsnorm_f32(x, gam, eps)
    elif kind == "bn_affine":
        y = x * gam + bet
    else:
        y = x.sum(-1) / cols
    with_y = tao.tao_bound_norm(code, x.cuda(), y.cuda(), gam.cuda(), bet.cuda(), eps=eps)
    without = tao.tao_bound_norm(code, x.cuda(), None, gam.cuda(), bet.cuda(), eps=eps)
    ok = ~torch.isnan(with_y)
    assert bool((without[ok] >= with_y[ok]).all())


@pytest.mark.parametrize("kind", ["layernorm", "rmsnorm"])
@pytest.mark.parametrize("rows,cols", [(1, 1), (5, 3), (300, 256), (17, 500), (130, 768), (257, 1024), (33, 1030),
                                       (40, 2048), (19, 4096), (6, 5000), (3, 8200), (4, 20000), (5000, 64), (0, 16)])
def test_norm_bound_checked_in_one_pass(tao, oracle_mod, kind, rows, cols):
    """tao_bound_check_norm: field for field the profile of tao_bound_norm followed by
    tao_check_and_profile, and of the oracle's check on the GPU's stored bound; a row without a bound
    (NaN), planted violations, with and without the affine scale, padded rows."""
    g = torch.Generator().manual_seed(rows * 131 + cols)
    ld = cols + (4 if cols % 8 == 0 and cols > 8 else 0)
    big = torch.randn((rows, ld), generator=g) * 2 + 0.5
    x = big[:, :cols]
    gam = 1 + 0.1 * torch.randn((cols,), generator=g)
    bet = 0.1 * torch.randn((cols,), generator=g)
    code = {"layernorm": 0, "rmsnorm": 1}[kind]
    eps = 1e-5
    xc = x.contiguous()
    y = (tao_inputs.layernorm_f32(xc, gam, bet, eps) if kind == "layernorm" else tao_inputs.rmsnorm_f32(xc, gam, eps)) if rows else xc.clone()
    claimed = tao_inputs.ulp_noise(g, y, max_ulps=2) if rows else y.clone()
    if rows > 2 and cols > 4:
        claimed[1, 2] = claimed[1, 2] * 1.01 + 0.1          # planted violation
        claimed[2, 0] = float("nan")
    if rows > 4 and cols > 4:
        big[3, 1] = float("nan")                            # a row without a bound
    pad = lambda t: torch.cat([t, torch.zeros((rows, ld - cols))], dim=1).cuda()[:, :cols] if ld != cols else t.cuda()
    xg, yg, cg = big.cuda()[:, :cols], pad(y), pad(claimed)
    for use_g in (True, False):
        gg, bb = (gam.cuda(), bet.cuda()) if use_g else (None, None)
        for alpha, eps_rel in ((1.0, 1e-12), (4.0, 1e-6)):
            fused = tao.tao_bound_check_norm(code, xg, yg, cg, gg, bb, eps=eps, alpha=alpha, eps_rel=eps_rel)
            if rows:
                tau = tao.tao_bound_norm(code, xg, yg, gg, bb, eps=eps)
            else:
                tau = torch.empty((0, cols), device="cuda")
            two = tao.tao_check_and_profile(cg.contiguous(), yg.contiguous(), tau.contiguous(), alpha=alpha, eps_rel=eps_rel)
            assert_profile_equal(fused, two, "%s %dx%d one pass vs two" % (kind, rows, cols))
            po = oracle_mod.check_and_profile(_np(claimed), _np(y), _np(tau), alpha=alpha, eps_rel=eps_rel)
            assert_profile_equal(fused, po, "%s %dx%d one pass vs oracle check" % (kind, rows, cols))
            assert fused["n"] == rows * cols
    if rows > 4 and cols > 4:
        assert fused["violations"] >= cols          # the whole NaN-bound row counts as violated


def test_norm_failure_rows_and_no_gamma(tao, oracle_mod):
    x = torch.full((3, 64), 3.0); x[1] = torch.arange(64.0); x[2, 5] = float("nan")
    y = torch.zeros((3, 64))
    t_or = oracle_mod.bound_norm(0, _np(x), y=_np(y), eps=1e-12)
    t_gpu = tao.tao_bound_norm(0, x.cuda(), y.cuda(), eps=1e-12)
    assert np.all(np.isnan(t_or[0])) and np.all(np.isnan(t_or[2]))
    assert_bound_parity(_np(t_gpu), t_or, "layernorm failure rows")
    t_or = oracle_mod.bound_norm(1, _np(x[1:2]), y=_np(y[1:2]), eps=1e-6)
    assert_bound_parity(_np(tao.tao_bound_norm(1, x[1:2].cuda(), y[1:2].cuda(), eps=1e-6)), t_or, "rmsnorm g=1")


@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 7), (64, 128), (100, 200), (513, 512), (257, 1000), (96, 2048),
                                       (40, 3000), (33, 4096), (9, 5000), (4, 20000), (5000, 64), (0, 16)])
def test_softmax_bound_checked_in_one_pass(tao, oracle_mod, rows, cols):
    """Field for field the profile of the two separate calls on the GPU, and of the oracle's check
    run on the GPU's stored bound; masked entries, a failing row and planted violations included."""
    g = torch.Generator().manual_seed(rows * 31 + cols)
    x = torch.randn((rows, cols), generator=g) * 3
    if rows > 2 and cols > 4:
        x[1, cols // 2:] = float("-inf")           # masked tail
        x[2, 0] = float("nan")                     # a row without a bound
    y = tao_inputs.softmax_f32(x) if rows else x.clone()
    claimed = tao_inputs.softmax_f32_reordered(g, x) if rows else x.clone()
    if rows > 4:
        claimed[3] = claimed[3] * 1.001            # planted violations
    xg, yg, cg = x.cuda(), y.cuda(), claimed.cuda()
    for alpha, eps in ((1.0, 1e-12), (2.5, 1e-6)):
        fused = tao.tao_bound_check_softmax(xg, yg, cg, alpha=alpha, eps_rel=eps)
        tau = tao.tao_bound_softmax(xg, yg)
        two = tao.tao_check_and_profile(cg, yg, tau, alpha=alpha, eps_rel=eps)
        assert_profile_equal(fused, two, "one pass vs two passes %dx%d" % (rows, cols))
        po = oracle_mod.check_and_profile(_np(claimed), _np(y), _np(tau), alpha=alpha, eps_rel=eps)
        assert_profile_equal(fused, po, "one pass vs oracle check %dx%d" % (rows, cols))
        assert fused["n"] == rows * cols
    if rows > 4 and cols > 4:
        assert fused["violations"] > 0


@pytest.mark.parametrize("M,N,K,batch", [(300, 200, 64, 2), (260, 390, 320, 2), (129, 70, 1100, 1)])
def test_matmul_check_with_padded_outputs(tao, M, N, K, batch):
    """y_ref, claimed and tau with a leading dimension beyond N and a batch stride beyond M ldy, through
    the C ABI: the same profile and the same bound as for contiguous tensors (short reductions take the
    epilogue route here, since the streaming check needs contiguous outputs)."""
    import paper_2510_16028_amd as binding
    g = torch.Generator().manual_seed(31 * M + N + K)
    A = torch.randn((batch, M, K), generator=g).cuda()
    W = torch.randn((batch, N, K), generator=g).cuda()
    y = torch.bmm(A, W.transpose(1, 2)).contiguous()
    claimed = (y * (1.0 + 3e-4 * torch.randn(y.shape, generator=g).cuda())).contiguous()
    tau_c = torch.empty_like(y)
    want = tao.tao_bound_check_linear(A, W, None, y, claimed, tau_out=tau_c)
    ldy, pad_rows = N + 8, 3
    sY = (M + pad_rows) * ldy
    def padded(t):
        buf = torch.full((batch, M + pad_rows, ldy), float("nan"), device="cuda")
        buf[:, :M, :N] = t
        return buf
    yp, cp = padded(y), padded(claimed)
    tp = torch.full((batch, M + pad_rows, ldy), -1.0, device="cuda")
    out = tao.new_profile_buffer(A.device)
    nbytes = tao.tao_bound_check_linear_workspace_bytes(M, N, K, batch, False)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    rc = binding.lib().tao_bound_check_linear(
        A.data_ptr(), W.data_ptr(), None, yp.data_ptr(), cp.data_ptr(), tp.data_ptr(),
        M, N, K, K, K, ldy, 0, batch, M * K, N * K, sY, 1.0, 1e-12, None, out.data_ptr(), ws.data_ptr(), nbytes, None)
    assert rc == 0
    torch.cuda.synchronize()
    got = tao.read_profile(out)
    assert_profile_equal(got, want, "padded outputs %s" % ((M, N, K, batch),))
    assert torch.equal(tp[:, :M, :N].contiguous().view(torch.int32), tau_c.view(torch.int32))
    assert bool((tp[:, :, N:] == -1.0).all()) and bool((tp[:, M:, :] == -1.0).all())      # nothing written outside


def test_split_tile_walk_against_one_workgroup_per_tile(tao):
    """Seeded shapes with short reductions and many tiles: the plain split bound walks its tiles
    (one workgroup per compute unit, slots beyond the ragged edges skipped), the checking launch
    takes one workgroup per slot; the bounds both store must be the same bits."""
    rng = np.random.default_rng(4711)
    for case in range(10):
        batch = int(rng.integers(4, 9))
        K = int(rng.integers(33, 1025))
        # at least 4 * 256 slots, so that the walk is taken on a 256-CU device: 280 to 450 tiles per
        # batch entry, ragged in both directions
        tm = int(rng.integers(10, 29)); tn = int(rng.integers(280, 450)) // tm + 1
        M = tm * 128 - int(rng.integers(0, 128)); N = tn * 128 - int(rng.integers(0, 128))
        assert batch * tm * tn >= 1100
        trans_w = bool(rng.integers(0, 2)); bias = bool(rng.integers(0, 2))
        g = torch.Generator().manual_seed(9000 + case)
        A = (torch.randn((batch, M, K), generator=g) * torch.exp(torch.randn((batch, M, 1), generator=g))).cuda()
        W = torch.randn((batch, K, N) if trans_w else (batch, N, K), generator=g).cuda()
        b = torch.randn((N,), generator=g).cuda() if bias else None
        walked = tao.tao_bound_linear_split(A, W, b, trans_w=trans_w)
        y = torch.zeros((batch, M, N), device="cuda")
        per_slot = torch.empty_like(y)
        tao.tao_bound_check_linear(A, W, b, y, y, trans_w=trans_w, tau_out=per_slot)
        torch.cuda.synchronize()
        same = torch.equal(walked.view(torch.int32), per_slot.view(torch.int32))
        assert same, "case %d: M=%d N=%d K=%d batch=%d trans_w=%s bias=%s" % (case, M, N, K, batch, trans_w, bias)
        print("case %d: M=%d N=%d K=%d batch=%d identical" % (case, M, N, K, batch), flush=True)


@pytest.mark.parametrize("M,N,K,bias,trans_w,batch", [
    (1, 1, 1, False, False, 1), (5, 7, 3, True, False, 1), (128, 128, 32, False, False, 1),
    (129, 257, 100, True, True, 1), (300, 200, 64, False, False, 3), (64, 640, 0, True, False, 1),
    (700, 390, 513, True, False, 2), (1024, 1152, 256, False, True, 1),     # 72 tiles: several per slot of the partials
    (4200, 1100, 96, True, False, 1),                                         # 297 tiles: more tiles than partial results
    (512, 384, 2048, True, False, 1), (300, 260, 1100, False, True, 2),       # reduction cut into parts: checked by the combining pass
    (0, 16, 8, False, False, 1),
    (2100, 1500, 100, True, False, 6), (1100, 2300, 40, False, True, 4),      # workgroups that walk several tiles
    (300, 260, 1000, True, False, 1),                                         # stored-bound route with the reduction cut into parts
])
def test_matmul_bound_checked_in_the_epilogue(tao, oracle_mod, M, N, K, bias, trans_w, batch):
    """tao_bound_check_linear: field for field the profile of tao_bound_linear_split followed by
    tao_check_and_profile, and of the oracle's check run on the stored bound; the optional tau
    output is bit-identical to the split path's; planted violations, NaN and infinite claims."""
    g = torch.Generator().manual_seed(M * 7 + N * 3 + K + batch)
    A = torch.randn((batch, M, K), generator=g)
    W = torch.randn((batch, K, N) if trans_w else (batch, N, K), generator=g)
    b = torch.randn((N,), generator=g) if bias else None
    if batch == 1:
        A, W = A[0], W[0]
    Wnk = W.transpose(-1, -2) if trans_w else W                      # [.., N, K]
    if K > 0:
        ref = A @ Wnk.transpose(-1, -2)
        claimed = tao_inputs.matmul_permuted_k(g, A, Wnk)            # another summation order
    else:
        ref = torch.zeros(A.shape[:-1] + (N,))
        claimed = ref.clone()
    if b is not None:
        ref = ref + b; claimed = claimed + b
    claimed = claimed.contiguous().clone()
    if M * N > 40:
        flat = claimed.reshape(-1)
        flat[3] = flat[3] * 1.01 + 1.0              # planted violation
        flat[7] = float("nan")
        flat[11] = float("inf")
    Ag, Wg, bg = A.cuda(), W.cuda(), None if b is None else b.cuda()
    rg, cg = ref.cuda().contiguous(), claimed.cuda().contiguous()
    tau = tao.tao_bound_linear_split(Ag, Wg, bg, trans_w=trans_w)
    # both routes of the entry point: its own choice (stored bound + streaming check up to K = 1024) and
    # the check in the matrix kernel's epilogue asked for by flag
    routes = (None, tao.FpModel(flags=tao.FLAG_CHECK_IN_EPILOGUE))
    for alpha, eps in ((1.0, 1e-12), (0.5, 1e-6)):
        two = tao.tao_check_and_profile(cg, rg, tau, alpha=alpha, eps_rel=eps)
        po = oracle_mod.check_and_profile(_np(claimed), _np(ref), _np(tau), alpha=alpha, eps_rel=eps)
        for model in routes:
            fused = tao.tao_bound_check_linear(Ag, Wg, bg, rg, cg, trans_w=trans_w, alpha=alpha, eps_rel=eps, model=model)
            assert_profile_equal(fused, two, "one call vs two passes %s" % ((M, N, K, batch, model is None),))
            assert_profile_equal(fused, po, "one call vs oracle check %s" % ((M, N, K, batch, model is None),))
            assert fused["n"] == batch * M * N
    # tau on request: the split path's bits
    for model in routes:
        tau2 = torch.full_like(tau, -1.0)
        again = tao.tao_bound_check_linear(Ag, Wg, bg, rg, cg, trans_w=trans_w, tau_out=tau2, model=model)
        assert bool((tau2.view(torch.int32) == tau.view(torch.int32)).all())
        assert_profile_equal(again, tao.tao_check_and_profile(cg, rg, tau), "with tau stored")
    if M * N > 40:
        assert again["violations"] >= 3 and again["nan_count"] >= 1


@pytest.mark.parametrize("M,N,K,bias,trans_w,batch,shared", [
    (1, 1, 1, False, False, 1, True), (129, 257, 49, True, False, 1, True), (130, 64, 601, False, True, 1, True),
    (33, 200, 48, True, True, 3, False), (96, 160, 320, False, False, 3, True), (5, 3, 0, True, False, 1, True),
    (2048, 1024, 4096, False, False, 1, True),      # reduction cut into parts: partial sums in the workspace
    (2100, 1500, 100, True, False, 6, False),       # tile walk
    (512, 384, 2048, True, False, 1, True), (300, 260, 1000, False, True, 2, False), (0, 16, 8, False, False, 1, True)])
def test_products_on_prepared_operand_images(tao, oracle_mod, M, N, K, bias, trans_w, batch, shared):
    """tao_split_operand + tao_bound_linear_images / tao_bound_check_linear_images: the bits of
    tao_bound_linear_split and the profile of tao_bound_check_linear, with the images built once and
    used twice (a second product on the same W image after other work has used the scratch memory)."""
    g = torch.Generator().manual_seed(M * 11 + N * 5 + K + batch)
    A = torch.randn((batch, M, K), generator=g)
    wb = 1 if shared else batch
    W = torch.randn((wb, K, N) if trans_w else (wb, N, K), generator=g)
    b = torch.randn((N,), generator=g).cuda() if bias else None
    if batch == 1:
        A = A[0]
    if wb == 1:
        W = W[0]
    Ag, Wg = A.cuda(), W.cuda()
    Wfull = Wg if (W.dim() == A.dim()) else Wg[None].expand((batch,) + tuple(Wg.shape))     # what the unprepared entry takes
    want = tao.tao_bound_linear_split(Ag, Wfull, b, trans_w=trans_w)
    A_img = tao.tao_split_operand(Ag) if M * K > 0 else Ag.new_empty(256, dtype=torch.uint8)
    W_img = tao.tao_split_operand(Wg, trans=trans_w) if N * K > 0 else Ag.new_empty(256, dtype=torch.uint8)
    sh = shared or batch == 1
    got = tao.tao_bound_linear_images(A_img, W_img, M, N, K, bias=b, batch=batch, shared_w=sh)
    assert torch.equal(got.view(torch.int32).reshape(-1), want.view(torch.int32).reshape(-1)), "images vs pre-pass inside the call"
    if M * N * batch > 0:
        assert_bound_parity(_np(got).reshape(-1), oracle_mod.bound_linear(_np(A), _np(Wfull), None if b is None else _np(b), trans_w=trans_w).reshape(-1),
                            "images vs oracle %s" % ((M, N, K, batch),))
    # the checked product on the same images
    Wnk = Wfull.transpose(-1, -2) if trans_w else Wfull
    ref = (Ag @ Wnk.transpose(-1, -2)) if K > 0 else torch.zeros(tuple(Ag.shape[:-1]) + (N,), device="cuda")
    if b is not None:
        ref = ref + b
    ref = ref.contiguous()
    claimed = tao_inputs.ulp_noise(torch.Generator(device="cuda").manual_seed(5), ref, max_ulps=2) if ref.numel() else ref.clone()
    if ref.numel() > 40:
        claimed.view(-1)[3] += 1.0
        claimed.view(-1)[9] = float("nan")
    for model in (None, tao.FpModel(flags=tao.FLAG_CHECK_IN_EPILOGUE)):
        one = tao.tao_bound_check_linear(Ag, Wfull, b, ref, claimed, trans_w=trans_w, alpha=2.0, model=model)
        tau2 = torch.full_like(want, -1.0)
        img = tao.tao_bound_check_linear_images(A_img, W_img, M, N, K, ref, claimed, bias=b, batch=batch, shared_w=sh, alpha=2.0,
                                                model=model, tau_out=tau2)
        assert_profile_equal(img, one, "checked product on images %s" % ((M, N, K, batch, model is None),))
        assert torch.equal(tau2.view(torch.int32).reshape(-1), want.view(torch.int32).reshape(-1))
    # the images are read only: a second product on them gives the same bits
    again = tao.tao_bound_linear_images(A_img, W_img, M, N, K, bias=b, batch=batch, shared_w=sh)
    assert torch.equal(again.view(torch.int32), got.view(torch.int32))


@pytest.mark.parametrize("M,N,K,bias,trans_w,batch", [
    (16640, 128, 1056, False, False, 1),     # 130 tiles, one column tile, 33 groups
    (16700, 200, 1088, True, True, 1),       # ragged rows and columns, two column tiles, W stored K x N
    (8900, 128, 1120, False, True, 2),       # batched (70 tiles each): the shape family of probabilities times values
])
def test_matmul_bound_with_the_a_operand_split_while_loaded(tao, oracle_mod, M, N, K, bias, trans_w, batch):
    """Products whose A operand serves one or two column tiles skip the pre-pass over A: the kernel
    cuts A into its pieces while loading it.  Same bits as the product on prepared images (which
    cannot take that route), parity with the oracle, and the checked variant's profile."""
    g = torch.Generator(device="cuda").manual_seed(M + N + K)
    A = torch.randn((batch, M, K), generator=g, device="cuda")
    W = torch.randn((batch, K, N) if trans_w else (batch, N, K), generator=g, device="cuda")
    A[0, 5, 7] = 0.0; A[0, 6, :] = 0.0                       # zeros and a zero row
    b = torch.randn((N,), generator=g, device="cuda") if bias else None
    if batch == 1:
        A, W = A[0], W[0]
    got = tao.tao_bound_linear_split(A, W, b, trans_w=trans_w)
    via_images = tao.tao_bound_linear_images(tao.tao_split_operand(A), tao.tao_split_operand(W, trans=trans_w), M, N, K,
                                             bias=b, batch=batch, shared_w=False)
    assert torch.equal(got.view(torch.int32).reshape(-1), via_images.view(torch.int32).reshape(-1))
    # the oracle on a sample of rows (the whole product would take it minutes)
    rows = torch.cat([torch.arange(0, 40), torch.arange(M - 140, M)])
    Ar = A[..., rows, :]
    t_or = oracle_mod.bound_linear(_np(Ar), _np(W), None if b is None else _np(b), trans_w=trans_w)
    assert_bound_parity(_np(got[..., rows, :]), t_or, "in-load split %s" % ((M, N, K, batch),))
    # checked in the epilogue (reductions beyond 1024): the profile of the two separate calls
    Wnk = W.transpose(-1, -2) if trans_w else W
    ref = A @ Wnk.transpose(-1, -2)
    if b is not None:
        ref = ref + b
    ref = ref.contiguous()
    claimed = tao_inputs.ulp_noise(g, ref, max_ulps=2)
    claimed.view(-1)[11] += 1.0
    one = tao.tao_bound_check_linear(A, W, b, ref, claimed, trans_w=trans_w)
    two = tao.tao_check_and_profile(claimed, ref, got)
    assert_profile_equal(one, two, "in-load split, checked in the epilogue")
    assert one["violations"] >= 1


def test_one_activation_image_feeds_several_projections(tao, oracle_mod):
    """An activation split once and multiplied with three weight images (the q / k / v pattern), and a
    weight image reused for a second activation."""
    g = torch.Generator().manual_seed(31)
    x = torch.randn((300, 520), generator=g).cuda()
    x_img = tao.tao_split_operand(x)
    ws = [torch.randn((n, 520), generator=g).cuda() * 0.02 for n in (520, 130, 129)]
    imgs = [tao.tao_split_operand(w) for w in ws]
    for w, wi in zip(ws, imgs):
        got = tao.tao_bound_linear_images(x_img, wi, 300, w.shape[0], 520)
        assert_bound_parity(_np(got), oracle_mod.bound_linear(_np(x), _np(w)), "shared activation image")
    x2 = torch.randn((77, 520), generator=g).cuda()
    got = tao.tao_bound_linear_images(tao.tao_split_operand(x2), imgs[0], 77, 520, 520)
    assert_bound_parity(_np(got), oracle_mod.bound_linear(_np(x2), _np(ws[0])), "shared weight image")


@pytest.mark.parametrize("N,C,spatial,G,affine", [
    (2, 32, (16, 16), 8, True),       # rows of 1024: cached, one wavefront per row
    (3, 12, (5, 7), 4, True),         # 105 columns: ragged, channel boundaries inside a vector
    (2, 6, (3,), 6, True),            # instance norm, three positions
    (1, 64, (32, 32), 32, False),     # 2048 columns, no affine
    (2, 128, (24, 24), 32, True),     # 2304 columns
    (1, 32, (64, 64), 2, True),       # 65536 columns: eight chunks per row
    (3, 10, (41, 43), 2, True),       # 8815 columns: a full chunk and a ragged one, unaligned rows
    (2, 4, (8193,), 4, False),        # one column beyond a chunk
    (16, 64, (48, 48), 32, True),     # 512 rows of 4608 ... and
    (64, 16, (70, 70), 8, True),      # 512 rows of 9800: long rows, one workgroup each (re-reading path)
    (4, 16, (1,), 1, True),           # one position, one group: LayerNorm over the channels
])
def test_groupnorm_shapes(tao, oracle_mod, N, C, spatial, G, affine):
    g = torch.Generator().manual_seed(N + 3 * C + G)
    x = torch.randn((N, C) + spatial, generator=g) * 2 + 0.5
    gam = (1 + 0.2 * torch.randn((C,), generator=g)) if affine else None
    bet = torch.randn((C,), generator=g) if affine else None
    y = torch.nn.functional.group_norm(x, G, gam, bet, eps=1e-5)
    t_or = oracle_mod.bound_groupnorm(_np(x), _np(y), G, None if gam is None else _np(gam),
                                      None if bet is None else _np(bet), eps=1e-5)
    t_gpu = tao.tao_bound_groupnorm(x.cuda(), y.cuda(), G, None if gam is None else gam.cuda(),
                                    None if bet is None else bet.cuda(), eps=1e-5)
    assert_bound_parity(_np(t_gpu), t_or, "groupnorm %s" % ((N, C, spatial, G),))
    # and the binary32 operator is inside the bound, against binary64
    y64 = torch.nn.functional.group_norm(x.double(), G, None if gam is None else gam.double(),
                                         None if bet is None else bet.double(), eps=float(np.float32(1e-5)))
    assert bool(((y.double() - y64).abs() <= t_gpu.cpu().double()).all())


@pytest.mark.parametrize("kind", ["gelu", "silu", "mul", "add", "relu"])
@pytest.mark.parametrize("n,offset", [(1, 0), (1023, 0), (4096, 1), ((1 << 20) + 3, 0)])
def test_act_shapes(tao, oracle_mod, kind, n, offset):
    g = torch.Generator().manual_seed(n + offset)
    x = (torch.randn((n + offset,), generator=g) * 4)[offset:]
    x2 = torch.randn((n + offset,), generator=g)[offset:]
    y = {"gelu": tao_inputs.gelu_f32, "silu": tao_inputs.silu_f32, "relu": torch.relu}.get(kind, None)
    y = y(x) if y else (x * x2 if kind == "mul" else x + x2)
    code = {"gelu": 0, "silu": 1, "mul": 2, "add": 3, "relu": 4}[kind]
    xg = x.cuda() if offset == 0 else torch.cat([torch.zeros(offset), x]).cuda()[offset:]
    yg = y.cuda() if offset == 0 else torch.cat([torch.zeros(offset), y]).cuda()[offset:]
    t_or = oracle_mod.bound_act(code, _np(x), _np(y), x2=_np(x2))
    t_gpu = tao.tao_bound_act(code, xg, yg, x2=x2.cuda())
    assert_bound_parity(_np(t_gpu), t_or, "%s n=%d" % (kind, n))


@pytest.mark.parametrize("kind", ["SUB", "DIV", "EXACT", "SQRT", "RSQRT", "EXP", "LOG", "SIN", "COS", "TANH",
                                  "POW", "SIGMOID"])
def test_one_step_kinds(tao, oracle_mod, kind):
    """tau depends on the verifier's output alone: any y exercises the formula; sizes with a
    ragged tail and a misaligned base, default and non-default accuracy constants."""
    code = getattr(oracle_mod, kind)
    assert code == getattr(tao, "ACT_" + kind)
    g = torch.Generator().manual_seed(code)
    for n, offset in ((1, 0), (4099, 1), ((1 << 18) + 3, 0)):
        y = (torch.randn((n + offset,), generator=g) * 10.0 ** torch.randint(-30, 30, (n + offset,), generator=g))[offset:]
        yg = torch.cat([torch.zeros(offset), y]).cuda()[offset:] if offset else y.cuda()
        for mo, mg in ((None, None),
                       (oracle_mod.Model(c_div=1.0, c_rsqrt=3.0, c_exp=1.0, c_log=5.0, c_sin=2.0, c_cos=6.0, c_tanh=2.0, c_pow=32.0),
                        tao.FpModel(c_div=1.0, c_rsqrt=3.0, c_exp=1.0, c_log=5.0, c_sin=2.0, c_cos=6.0, c_tanh=2.0, c_pow=32.0))):
            t_or = oracle_mod.bound_act(code, None, _np(y), model=mo)
            t_gpu = tao.tao_bound_act(code, None, yg, model=mg)
            assert_bound_parity(_np(t_gpu), t_or, "%s n=%d" % (kind, n))


@pytest.mark.parametrize("kind", ["GELU_ERF", "GELU_TANH", "SILU", "MUL", "ADD", "RELU", "DIV", "EXP", "EXACT", "SIGMOID"])
def test_elementwise_bound_checked_in_one_pass(tao, oracle_mod, kind):
    """tao_bound_check_act: field for field the profile of tao_bound_act followed by
    tao_check_and_profile on the GPU, and of the oracle's check on the GPU's stored bound; ragged
    sizes, a misaligned base, planted violations, NaN and infinite claims."""
    code = getattr(oracle_mod, kind)
    g = torch.Generator().manual_seed(code + 77)
    for n, offset in ((0, 0), (1, 0), (4099, 1), ((1 << 20) + 3, 0), (5 * (1 << 20), 0)):
        x = (torch.randn((n + offset,), generator=g) * 3)[offset:]
        x2 = torch.randn((n + offset,), generator=g)[offset:]
        ref = {"GELU_ERF": tao_inputs.gelu_f32, "GELU_TANH": lambda v: torch.nn.functional.gelu(v, approximate="tanh"),
               "SILU": tao_inputs.silu_f32, "RELU": torch.relu, "EXP": torch.exp, "SIGMOID": torch.sigmoid,
               "EXACT": lambda v: v.clone(), "MUL": lambda v: v * x2, "ADD": lambda v: v + x2, "DIV": lambda v: v / x2}[kind](x)
        claimed = tao_inputs.ulp_noise(g, ref, max_ulps=2) if n else ref.clone()
        if n > 100:
            claimed[5] = claimed[5] * 1.001 + 1e-3
            claimed[17] = float("nan")
            claimed[40] = float("inf")
        dev = lambda t: (torch.cat([torch.zeros(offset), t]).cuda()[offset:] if offset else t.cuda())
        xg, yg, cg = dev(x), dev(ref), dev(claimed)
        needs_x = kind.startswith("GELU")
        for alpha, eps in ((1.0, 1e-12), (3.0, 1e-6)):
            fused = tao.tao_bound_check_act(code, xg if needs_x else None, yg, cg, alpha=alpha, eps_rel=eps)
            tau = tao.tao_bound_act(code, xg if needs_x else None, yg) if n else torch.empty(0, device="cuda")
            two = tao.tao_check_and_profile(cg, yg, tau, alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, two, "%s n=%d one pass vs two" % (kind, n))
            po = oracle_mod.check_and_profile(_np(claimed), _np(ref), _np(tau), alpha=alpha, eps_rel=eps)
            assert_profile_equal(fused, po, "%s n=%d one pass vs oracle check" % (kind, n))
            assert fused["n"] == n
        if n > 100:
            assert fused["violations"] >= 2 and fused["nan_count"] >= 1


def test_gelu_tanh_shapes_and_range(tao, oracle_mod):
    code = oracle_mod.GELU_TANH
    for n, offset in ((1, 0), (1023, 0), (4096, 1), ((1 << 20) + 3, 0)):
        g = torch.Generator().manual_seed(n + offset)
        x = (torch.randn((n + offset,), generator=g) * 4)[offset:]
        y = torch.nn.functional.gelu(x, approximate="tanh")
        xg = torch.cat([torch.zeros(offset), x]).cuda()[offset:] if offset else x.cuda()
        yg = torch.cat([torch.zeros(offset), y]).cuda()[offset:] if offset else y.cuda()
        assert_bound_parity(_np(tao.tao_bound_act(code, xg, yg)), oracle_mod.bound_act(code, _np(x), _np(y)), "gelu tanh n=%d" % n)
    x = torch.cat([torch.linspace(-40, 40, 200001),
                   torch.tensor([0.0, -0.0, 1e-30, -1e-30, 1e-45, 38.5, -38.5, 1e20, -3e38, float("inf"), float("nan")])])
    y = torch.nn.functional.gelu(x, approximate="tanh")
    t_or = oracle_mod.bound_act(code, _np(x), _np(y))
    assert_bound_parity(_np(tao.tao_bound_act(code, x.cuda(), y.cuda())), t_or, "gelu tanh range")
    # the honest binary32 result is inside the bound, against binary64
    y64 = torch.nn.functional.gelu(x[:200001].double(), approximate="tanh")
    assert bool(((y[:200001].double() - y64).abs() <= torch.from_numpy(t_or[:200001]).double()).all())
    m_o, m_g = oracle_mod.Model(c_tanh=9.0, flags=0), tao.FpModel(c_tanh=9.0)
    assert_bound_parity(_np(tao.tao_bound_act(code, x.cuda(), y.cuda(), model=m_g)),
                        oracle_mod.bound_act(code, _np(x), _np(y), model=m_o), "gelu tanh c_tanh=9")


@pytest.mark.parametrize("rows,d,inner,npos,interleaved", [
    (64, 128, 4, 16, False), (64, 128, 1, 64, True), (37, 6, 3, 5, False), (37, 6, 1, 7, True),
    (5, 2, 1, 1, False), (1000, 64, 8, 125, False), (33, 20, 2, 3, True), (16384, 128, 32, 512, False)])
def test_rope_shapes(tao, oracle_mod, rows, d, inner, npos, interleaved):
    g = torch.Generator().manual_seed(rows + d)
    x = torch.randn((rows, d), generator=g) * 3
    pos = torch.arange(npos, dtype=torch.float64)[:, None]
    freq = 1e6 ** (-torch.arange(d // 2, dtype=torch.float64) / max(d // 2, 1))[None, :]
    cs, sn = torch.cos(pos * freq).float(), torch.sin(pos * freq).float()
    t_or = oracle_mod.bound_rope(_np(x), _np(cs), _np(sn), inner=inner, interleaved=interleaved)
    t_gpu = tao.tao_bound_rope(x.cuda(), cs.cuda(), sn.cuda(), inner=inner, interleaved=interleaved)
    assert_bound_parity(_np(t_gpu), t_or, "rope %s" % ((rows, d, inner, npos, interleaved),))
    # misaligned base: the scalar path
    xo = torch.cat([torch.zeros(1), x.reshape(-1)]).cuda()[1:].reshape(rows, d)
    assert_bound_parity(_np(tao.tao_bound_rope(xo, cs.cuda(), sn.cuda(), inner=inner, interleaved=interleaved)), t_or, "rope misaligned")
    # checked in the same pass: the profile of the two separate calls, and of the oracle's check on the stored bound
    rot = torch.empty_like(x)
    tpos = (torch.arange(rows) // inner) % npos
    c_, s_ = cs[tpos], sn[tpos]
    if interleaved:
        xa, xb = x[:, 0::2], x[:, 1::2]
        rot[:, 0::2], rot[:, 1::2] = xa * c_ - xb * s_, xb * c_ + xa * s_
    else:
        xa, xb = x[:, : d // 2], x[:, d // 2:]
        rot[:, : d // 2], rot[:, d // 2:] = xa * c_ - xb * s_, xb * c_ + xa * s_
    claimed = tao_inputs.ulp_noise(g, rot, max_ulps=1)
    claimed[0, 0] = claimed[0, 0] + 1.0
    fused = tao.tao_bound_check_rope(x.cuda(), cs.cuda(), sn.cuda(), rot.cuda(), claimed.cuda(), inner=inner,
                                     interleaved=interleaved, alpha=2.0)
    two = tao.tao_check_and_profile(claimed.cuda(), rot.cuda(), t_gpu, alpha=2.0)
    assert_profile_equal(fused, two, "rope one pass vs two")
    assert_profile_equal(fused, oracle_mod.check_and_profile(_np(claimed), _np(rot), _np(t_gpu), alpha=2.0), "rope one pass vs oracle check")
    assert fused["violations"] >= 1 and fused["n"] == rows * d
    mo, mg = oracle_mod.Model(flags=1, mode=1), tao.FpModel(flags=tao.FLAG_UNDERFLOW_TERMS, mode=1)
    assert_bound_parity(_np(tao.tao_bound_rope(x.cuda(), cs.cuda(), sn.cuda(), inner=inner, interleaved=interleaved, model=mg)),
                        oracle_mod.bound_rope(_np(x), _np(cs), _np(sn), inner=inner, interleaved=interleaved, model=mo), "rope flags")


def test_rope_accepts_a_real_rotation(tao, oracle_mod):
    """Binary32 rotate-half RoPE against binary64: every error inside the GPU's bound."""
    g = torch.Generator().manual_seed(4)
    T, Hd, d = 256, 8, 128
    x = torch.randn((T, Hd, d), generator=g)
    pos = torch.arange(T, dtype=torch.float64)[:, None]
    freq = 1e6 ** (-torch.arange(d // 2, dtype=torch.float64) / (d // 2))[None, :]
    cs, sn = torch.cos(pos * freq).float(), torch.sin(pos * freq).float()
    def rot(x, c, s):
        a, b = x[..., :d // 2], x[..., d // 2:]
        return torch.cat([a * c[:, None, :] - b * s[:, None, :], b * c[:, None, :] + a * s[:, None, :]], dim=-1)
    y32, y64 = rot(x, cs, sn), rot(x.double(), cs.double(), sn.double())
    tau = tao.tao_bound_rope(x.cuda(), cs.cuda(), sn.cuda(), inner=Hd)
    assert bool(((y32.double() - y64).abs() <= tau.cpu().double()).all())


def test_gelu_wide_range(tao, oracle_mod):
    x = torch.cat([torch.linspace(-40, 40, 200001), torch.tensor([0.0, -0.0, 1e-30, -1e-30, 38.5, -38.5])])
    y = tao_inputs.gelu_f32(x)
    assert_bound_parity(_np(tao.tao_bound_act(0, x.cuda(), y.cuda())), oracle_mod.bound_act(0, _np(x), _np(y)), "gelu range")


@pytest.mark.parametrize("n,offset", [(0, 0), (1, 0), (5, 0), (1000, 1), ((1 << 20) + 3, 0), (300001, 3)])
def test_check_sizes(tao, oracle_mod, n, offset):
    c, r, t = tao_inputs.check_triplet("cpu", seed=1000 + n, n=n + offset)
    c, r, t = c[offset:], r[offset:], t[offset:]
    cg, rg, tg = [torch.cat([torch.zeros(offset), v]).cuda()[offset:] if offset else v.cuda() for v in (c, r, t)]
    for alpha, eps in ((1.0, 1e-12), (0.5, 0.0), (3.0, 1e-3)):
        pg = tao.tao_check_and_profile(cg, rg, tg, alpha=alpha, eps_rel=eps)
        po = oracle_mod.check_and_profile(_np(c), _np(r), _np(t), alpha=alpha, eps_rel=eps)
        assert_profile_equal(pg, po, "check n=%d alpha=%g" % (n, alpha))
    if n > 1000:
        assert 0 < po["violations"] < n


def test_check_special_values_and_clusters(tao, oracle_mod):
    ref = torch.tensor([1.0, 0.0, 0.0, float("nan"), 1.0, float("inf"), 3e38, 1e-40, -2.0])
    claimed = torch.tensor([1.0, 0.0, 1.0, 1.0, float("nan"), float("inf"), -3e38, 0.0, -2.0000002])
    tau = torch.tensor([0.0, 0.0, 2.0, 1.0, 1.0, 1.0, float("inf"), 1e-38, float("nan")])
    for eps in (0.0, 1e-12, 1e10):
        pg = tao.tao_check_and_profile(claimed.cuda(), ref.cuda(), tau.cuda(), eps_rel=eps)
        po = oracle_mod.check_and_profile(_np(claimed), _np(ref), _np(tau), eps_rel=eps)
        assert_profile_equal(pg, po, "special eps=%g" % eps)
    # every element in one bin (worst case for the LDS histogram), and two-call reuse of buffers
    n = 1 << 18
    ref = torch.ones(n); claimed = torch.full((n,), 1.0 + 2.0 ** -12); tau = torch.full((n,), 1e-3)
    for _ in range(2):
        pg = tao.tao_check_and_profile(claimed.cuda(), ref.cuda(), tau.cuda(), eps_rel=0.0)
        po = oracle_mod.check_and_profile(_np(claimed), _np(ref), _np(tau), eps_rel=0.0)
        assert_profile_equal(pg, po, "single bin")
    assert po["hist"][(127 - 12) << 3] == n


def _assert_error_profile_equal(pg, po, what):
    for k in ("n", "nan_count", "offending"):
        assert pg[k] == po[k], (what, k, pg[k], po[k])
    for k in ("hist_abs", "hist_rel", "abs_bin", "rel_bin"):
        assert np.array_equal(pg[k], po[k]), (what, k)
    for k in ("abs_p", "rel_p"):
        assert np.array_equal(pg[k].view(np.uint32), po[k].view(np.uint32)), (what, k, pg[k], po[k])
    for k in ("max_abs", "max_rel", "p_max"):
        a, b = np.float64(pg[k]), np.float64(po[k])
        assert (np.isnan(a) and np.isnan(b)) or a == b, (what, k, a, b)


@pytest.mark.parametrize("n,offset", [(0, 0), (1, 0), (7, 0), (1000, 1), ((1 << 20) + 3, 0), (300001, 3)])
def test_profile_errors_sizes(tao, oracle_mod, n, offset):
    """Error profiles on the 22-point grid and the selection statistic: bit-exact against the oracle
    (integer histograms and ranks, IEEE binary64 per element and for the threshold quotients)."""
    c, r, _ = tao_inputs.check_triplet("cpu", seed=2000 + n, n=n + offset)
    c, r = c[offset:], r[offset:]
    cg, rg = [torch.cat([torch.zeros(offset), v]).cuda()[offset:] if offset else v.cuda() for v in (c, r)]
    for eps in (1e-12, 0.0, 1e-3):
        pg = tao.tao_profile_errors(cg, rg, eps_rel=eps)
        po = oracle_mod.profile_errors(_np(c), _np(r), eps_rel=eps)
        _assert_error_profile_equal(pg, po, "errors n=%d eps=%g" % (n, eps))
        assert np.isnan(pg["p_max"]) and pg["offending"] == 0
    if n == 0:
        return
    # thresholds = alpha x the profile itself (threshold construction of Sec. 3.2, alpha = 3), then one
    # entry pushed below the observed percentile
    base = oracle_mod.profile_errors(_np(c), _np(r))
    ta = (3 * base["abs_p"]).astype(np.float32); tr = (3 * base["rel_p"]).astype(np.float32)
    for tweak in (False, True):
        if tweak:
            tr[10] = base["rel_p"][10] / np.float32(2)
        pg = tao.tao_profile_errors(cg, rg, thr_abs=torch.from_numpy(ta).cuda(), thr_rel=torch.from_numpy(tr).cuda())
        po = oracle_mod.profile_errors(_np(c), _np(r), thr_abs=ta, thr_rel=tr)
        _assert_error_profile_equal(pg, po, "errors n=%d thresholds tweak=%s" % (n, tweak))
    if n > 1000 and base["rel_p"][10] > 0:
        assert po["offending"] == 1 and po["p_max"] == 2.0


def test_profile_errors_special_values(tao, oracle_mod):
    ref = torch.tensor([1.0, 0.0, 0.0, float("nan"), 1.0, float("inf"), 3e38, 1e-40, -2.0, 2.0])
    claimed = torch.tensor([1.0, 0.0, 1.0, 1.0, float("nan"), float("inf"), -3e38, 0.0, -2.0000002, float("inf")])
    for eps in (0.0, 1e-12, 1e10):
        pg = tao.tao_profile_errors(claimed.cuda(), ref.cuda(), eps_rel=eps)
        po = oracle_mod.profile_errors(_np(claimed), _np(ref), eps_rel=eps)
        _assert_error_profile_equal(pg, po, "special eps=%g" % eps)
    # identical outputs with zero thresholds: every quotient is 0/0 or 0/thr
    z = torch.randn(5000)
    ta = np.zeros(22, np.float32); tr = np.ones(22, np.float32)
    pg = tao.tao_profile_errors(z.cuda(), z.cuda(), thr_abs=torch.from_numpy(ta).cuda(), thr_rel=torch.from_numpy(tr).cuda())
    po = oracle_mod.profile_errors(_np(z), _np(z), thr_abs=ta, thr_rel=tr)
    _assert_error_profile_equal(pg, po, "identical")
    assert pg["p_max"] == 0.0 and pg["max_abs"] == 0.0
    # every element in one bin, twice with the same buffers
    n = 1 << 18
    ref = torch.ones(n); claimed = torch.full((n,), 1.0 + 2.0 ** -12)
    for _ in range(2):
        pg = tao.tao_profile_errors(claimed.cuda(), ref.cuda(), eps_rel=0.0)
        po = oracle_mod.profile_errors(_np(claimed), _np(ref), eps_rel=0.0)
        _assert_error_profile_equal(pg, po, "single bin")


def test_calibration_envelope_and_thresholds(tao, oracle_mod):
    """Calibration loop of Sec. 3.2 on the device: profiles of several runs -> envelope -> thresholds,
    bit-exact against the oracle; the thresholds then accept every calibration run."""
    import ctypes
    rng = np.random.Generator(np.random.Philox(48))
    ref = torch.from_numpy(rng.standard_normal(70001).astype(np.float32))
    runs = [(ref * (1 + s * torch.from_numpy(rng.standard_normal(70001).astype(np.float32)))) for s in (1e-6, 2e-6, 5e-7, 3e-6, 1e-6)]
    size = ctypes.sizeof(tao.ErrorProfile)
    bufs = torch.empty((len(runs), size), dtype=torch.uint8, device="cuda")
    for i, c in enumerate(runs):
        tao.tao_profile_errors(c.cuda(), ref.cuda(), out=bufs[i], readback=False)
    for alpha in (3.0, 1.0, 2.5):
        ea, er, ta, tr = [_np(t) for t in tao.tao_calibrate_thresholds(bufs, alpha=alpha)]
        profs = [oracle_mod.profile_errors(_np(c), _np(ref)) for c in runs]
        oa, orr, ota, otr = oracle_mod.calibrate_thresholds([(p["abs_p"], p["rel_p"]) for p in profs], alpha=alpha)
        for g, o in ((ea, oa), (er, orr), (ta, ota), (tr, otr)):
            assert np.array_equal(g.view(np.uint32), o.view(np.uint32))
    ea, er, ta, tr = tao.tao_calibrate_thresholds(bufs, alpha=3.0)
    for c in runs:
        p = tao.tao_profile_errors(c.cuda(), ref.cuda(), thr_abs=ta, thr_rel=tr)
        assert p["offending"] == 0 and p["p_max"] <= 1 / 3 + 1e-7
    bad = ref * (1 + 3e-5 * torch.from_numpy(rng.standard_normal(70001).astype(np.float32)))
    assert tao.tao_profile_errors(bad.cuda(), ref.cuda(), thr_abs=ta, thr_rel=tr)["offending"] == 1
    # a single run and NaN handling: a run whose profile is NaN at the top (NaN errors) is skipped there
    c = runs[0].clone(); c[5] = float("nan")
    tao.tao_profile_errors(c.cuda(), ref.cuda(), out=bufs[0], readback=False)
    ea, er, ta, tr = [_np(t) for t in tao.tao_calibrate_thresholds(bufs[:2], alpha=3.0)]
    profs = [oracle_mod.profile_errors(_np(c), _np(ref)), oracle_mod.profile_errors(_np(runs[1]), _np(ref))]
    oa, orr, ota, otr = oracle_mod.calibrate_thresholds([(p["abs_p"], p["rel_p"]) for p in profs], alpha=3.0)
    assert np.isnan(profs[0]["rel_p"][-1]) and not np.isnan(orr[-1])
    for g, o in ((ea, oa), (er, orr), (ta, ota), (tr, otr)):
        assert np.array_equal(g.view(np.uint32), o.view(np.uint32))
