#!/usr/bin/env python3
"""Benchmark of the tolerance engine's hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: for
every traced operator of a Qwen3-8B-shaped decoder layer (hidden 4096,
intermediate 12288, 32 q / 8 kv heads, head_dim 128, seq 2048) compute the
bound tensor tau (linear, softmax, RMSNorm, SiLU, Mul, Add, rotary kinds) and run
the check + relative-error profile of the claimed output against the re-executed
one.  All inputs are resident in HBM before the timed region.  The weights of the
layer are committed constants: their BF16 images are prepared once, before the
timed region; every activation is split again in every step, inside it.

Prints ONE JSON line.  `value` = bytes of claimed operator output verified per
second (4 bytes per element that went through bound + check) on configuration 3.
`roofline` is for the dominant kernel (the MFMA |A||W| bound), from HIP events
recorded around its launches inside the timed region.  `configs` holds the same
measurement for the other configurations (1, 2, 4 and the 8192^3 stress case),
`kernels` the individual kernels, also the bound kernels that store tau at
100 M elements and more.  `cpu_baseline` times the CPU oracle on a row sample of
configuration 3.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch of the dominant kernel, measured offline with two rocprofv3 counter passes
# over this same command (FETCH_SIZE, WRITE_SIZE, scaled by a copy kernel); the summary is kept
# as text next to the other profiles and only its one figure is read here.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "bench_c3_hbm_traffic.md")


def measured_traffic(kernel):
    """Bytes per launch recorded in the committed counter summary, or None."""
    import re
    try:
        text = open(TRAFFIC_SUMMARY).read()
    except OSError:
        return None
    m = re.search(r"^%s traffic bytes per launch: (\d+)$" % re.escape(kernel), text, re.M)
    return int(m.group(1)) if m else None


_NORM = {"layernorm": 0, "rmsnorm": 1, "bn_affine": 2, "sum": 3, "mean": 4}
_ACT = {"gelu": 0, "silu": 1, "mul": 2, "add": 3, "relu": 4}
# algorithmic HBM bytes per output element of the streaming bound kernels (inputs read once,
# tau written once)
_STREAM_BYTES = {"softmax": 12, "layernorm": 12, "rmsnorm": 12, "bn_affine": 12, "gelu": 12,
                 "silu": 8, "mul": 8, "add": 8, "rope": 8}
# the same with the check in the same pass: inputs and the claimed output read once, nothing written
_FUSED_BYTES = {"softmax": 12, "gelu": 12, "silu": 8, "mul": 8, "add": 8, "relu": 8, "layernorm": 12, "rmsnorm": 12,
                "rope": 12}


class PlannedOp:
    """One operator with every buffer preallocated; run() only enqueues kernels.

    images: the plan's table of activation images (key: the activation's address); the first operator
    that multiplies an activation splits it, in every step, and later operators of the step reuse the
    image (the q / k / v and the gate / up projections share theirs)."""

    def __init__(self, tao, torch, op, images, use_split=True, use_fused=True, prepared=True):
        self.tao, self.op, self.kind, self.name = tao, op, op.kind, op.name
        self.claimed = op.claimed.contiguous()
        self.y_ref = op.y_ref.contiguous()
        self.tau = torch.empty_like(self.y_ref)
        self.prof = tao.new_profile_buffer(self.y_ref.device)
        self.n = self.y_ref.numel()
        a = op.args
        self.split = self.fused = self.prepared = self.conv = False
        self.owns_image = False
        if self.kind == "linear":
            A, W = a["A"], a["W"]
            K = A.shape[-1]
            self.flops = 2.0 * self.n * K
            self.min_bytes = 4.0 * (A.numel() + W.numel() + self.n)
            batch = A.shape[0] if A.dim() == 3 else 1
            M, N = self.y_ref.shape[-2], self.y_ref.shape[-1]
            self.dims = (M, N, K, batch)
            self.conv = "conv" in op.attrs
            if self.conv:
                cv = op.attrs["conv"]
                # the convolution on the BF16 matrix cores (patch matrix gathered and split while loaded),
                # where the library serves the shape; else its FP32 implicit-GEMM kernel
                self.split = use_split and tao.tao_conv2d_split_supported(cv["x"].shape, cv["w"].shape, 1, cv["padding"], 1)
                self.fused = self.split and use_fused
                if self.split:
                    need = tao.lib().tao_conv2d_split_workspace_bytes(*cv["x"].shape, cv["w"].shape[0], cv["w"].shape[1], cv["w"].shape[2],
                                                                      1, 1, cv["padding"], cv["padding"], 1, 1, 1)
                    self.ws = torch.empty(max(int(need), 256), dtype=torch.uint8, device=A.device)
                self.bound_events, self.check_events = [], []
                return
            # the library's own rule picks the BF16-split or the FP32 matrix-core path per shape
            self.split = use_split and tao.tao_linear_split_preferred(M, N, K, batch)
            # ... and there the check runs in the matrix kernel's epilogue (tau is never stored)
            # (short reductions: the library itself would store the bound and run the streaming check; the
            # benchmark makes the two calls itself so that the matmul figure times the matmul kernels alone)
            self.fused = self.split and use_fused and tao.tao_bound_check_linear_in_epilogue(M, N, K, batch)
            self.prepared = self.split and prepared and bool(op.attrs.get("weight")) and not op.attrs.get("trans_w", 0)
            if self.prepared:
                self.w_image = tao.tao_split_operand(W)            # once: the weights do not change
                key = (A.data_ptr(), tuple(A.shape))
                if key not in images:
                    images[key] = torch.empty(tao.tao_split_image_bytes(M, K, batch), dtype=torch.uint8, device=A.device)
                    self.owns_image = True
                self.a_image = images[key]
                need = (tao.lib().tao_check_linear_images_workspace_bytes if self.fused
                        else tao.lib().tao_linear_images_workspace_bytes)(M, N, K, batch)
                self.ws = torch.empty(max(int(need), 256), dtype=torch.uint8, device=A.device)
            elif self.split:
                shared = W.dim() == 2 or batch == 1
                need = (tao.tao_bound_check_linear_workspace_bytes if self.fused
                        else tao.tao_linear_split_workspace_bytes)(M, N, K, batch, shared)
                self.ws = torch.empty(need, dtype=torch.uint8, device=A.device)
        else:
            self.flops = 0.0
            self.min_bytes = 0.0
            # element-wise operators and softmax: bound and check in one streaming pass
            self.fused = use_fused and self.kind in _FUSED_BYTES
            if self.fused:
                self.ws = torch.empty(tao.tao_check_workspace_bytes(self.n), dtype=torch.uint8, device=self.y_ref.device)
        self.bound_events, self.check_events = [], []

    @property
    def path(self):
        if self.conv:
            return ("bf16_split (patch matrix gathered while loaded)" + ("+check" if self.fused else "")) if self.split else "fp32 (implicit patch matrix)"
        if not self.split:
            return "fp32"
        return "bf16_split" + ("+prepared_w" if self.prepared else "") + ("+check" if self.fused else "")

    def bound(self):
        tao, a, op = self.tao, self.op.args, self.op
        if self.kind == "linear" and self.conv:
            cv = op.attrs["conv"]
            if self.split:
                tao.tao_bound_conv2d_split(cv["x"], cv["w"], None, 1, cv["padding"], 1, out=self.tau.view(self.conv_shape()), ws=self.ws)
            else:
                tao.tao_bound_conv2d(cv["x"], cv["w"], None, 1, cv["padding"], 1, out=self.tau.view(self.conv_shape()))
        elif self.kind == "linear" and self.prepared:
            M, N, K, batch = self.dims
            if self.owns_image:
                tao.tao_split_operand(a["A"], out=self.a_image)
            tao.tao_bound_linear_images(self.a_image, self.w_image, M, N, K, bias=a.get("bias"), batch=batch, out=self.tau, ws=self.ws)
        elif self.kind == "linear" and self.split:
            tao.tao_bound_linear_split(a["A"], a["W"], a.get("bias"), trans_w=bool(op.attrs.get("trans_w", 0)),
                                       out=self.tau, ws=self.ws)
        elif self.kind == "linear":
            tao.tao_bound_linear(a["A"], a["W"], a.get("bias"), trans_w=bool(op.attrs.get("trans_w", 0)), out=self.tau)
        elif self.kind == "softmax":
            tao.tao_bound_softmax(a["x"], self.y_ref, out=self.tau)
        elif self.kind in ("layernorm", "rmsnorm"):
            tao.tao_bound_norm(_NORM[self.kind], a["x"], self.y_ref, a.get("gamma"), a.get("beta"),
                               eps=op.attrs["eps"], out=self.tau)
        elif self.kind == "bn_affine":
            tao.tao_bound_norm(2, a["x"], self.y_ref, a["scale"], a["shift"], out=self.tau)
        elif self.kind == "rope":
            tao.tao_bound_rope(a["x"], a["cos"], a["sin"], inner=op.attrs["inner"], out=self.tau)
        else:
            tao.tao_bound_act(_ACT[self.kind], a.get("x"), self.y_ref, x2=a.get("x2"), out=self.tau)

    def conv_shape(self):
        x = self.op.attrs["conv"]["x"]                      # [B, H, W, C], 3x3 / stride 1 / pad 1: same extent
        return (x.shape[0], x.shape[1], x.shape[2], self.tau.shape[-1])

    def check(self):
        self.tao.tao_check_and_profile(self.claimed, self.y_ref, self.tau, out=self.prof, readback=False)

    def bound_and_check(self):
        a, op = self.op.args, self.op
        if self.kind == "softmax":
            self.tao.tao_bound_check_softmax(a["x"], self.y_ref, self.claimed, out=self.prof, ws=self.ws, readback=False)
            return
        if self.kind in ("layernorm", "rmsnorm"):
            self.tao.tao_bound_check_norm(_NORM[self.kind], a["x"], self.y_ref, self.claimed, a.get("gamma"), a.get("beta"),
                                          eps=op.attrs["eps"], out=self.prof, ws=self.ws, readback=False)
            return
        if self.kind == "rope":
            self.tao.tao_bound_check_rope(a["x"], a["cos"], a["sin"], self.y_ref, self.claimed, inner=op.attrs["inner"],
                                          out=self.prof, ws=self.ws, readback=False)
            return
        if self.kind != "linear":
            self.tao.tao_bound_check_act(_ACT[self.kind], a.get("x"), self.y_ref, self.claimed, x2=a.get("x2"),
                                         out=self.prof, ws=self.ws, readback=False)
            return
        if self.conv:
            cv = op.attrs["conv"]
            self.tao.tao_bound_check_conv2d(cv["x"], cv["w"], None, self.y_ref, self.claimed, 1, cv["padding"], 1,
                                            out=self.prof, ws=self.ws, readback=False)
            return
        if self.prepared:
            M, N, K, batch = self.dims
            if self.owns_image:
                self.tao.tao_split_operand(a["A"], out=self.a_image)
            self.tao.tao_bound_check_linear_images(self.a_image, self.w_image, M, N, K, self.y_ref, self.claimed, bias=a.get("bias"),
                                                   batch=batch, out=self.prof, ws=self.ws, readback=False)
            return
        self.tao.tao_bound_check_linear(a["A"], a["W"], a.get("bias"), self.y_ref, self.claimed,
                                        trans_w=bool(op.attrs.get("trans_w", 0)), out=self.prof, ws=self.ws,
                                        readback=False)

    def run(self, torch, record):
        if self.fused:
            if record:
                e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                e[0].record(); self.bound_and_check(); e[1].record()
                self.bound_events.append((e[0], e[1]))
            else:
                self.bound_and_check()
            return
        if record:
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(); self.bound(); e[1].record(); self.check(); e[2].record()
            self.bound_events.append((e[0], e[1])); self.check_events.append((e[1], e[2]))
        else:
            self.bound(); self.check()


def _ms(pairs):
    return [a.elapsed_time(b) for a, b in pairs]


def _event_time(torch, fn, reps, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record(); fn(); b.record()
    torch.cuda.synchronize()
    return sum(_ms(ev)) / reps


def shader_clock_under(torch, fn, samples=3):
    """The shader clock (MHz) rocm-smi reports while `fn` keeps the GPU busy, or None if it cannot be read.
    (The matrix cores' peaks are quoted at 2.4 GHz; the chip lowers its clock under dense BF16 MFMA work.)
    rocm-smi takes a few hundred milliseconds to start: launches are queued, a few at a time, until it has
    answered, so the clock it reads is the one under load."""
    import re, subprocess
    try:
        seen = []
        for _ in range(samples):
            for _ in range(4):
                fn()
            torch.cuda.synchronize()
            proc = subprocess.Popen(["rocm-smi", "--showclocks"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
            t0 = time.perf_counter()
            while proc.poll() is None and time.perf_counter() - t0 < 10.0:
                for _ in range(4):
                    fn()
                torch.cuda.synchronize()
            if proc.poll() is None:
                proc.kill()
                proc.communicate()
                return None
            m = re.search(r"sclk clock level: \d+: \((\d+)Mhz\)", proc.communicate()[0])
            if m:
                seen.append(int(m.group(1)))
        return (sum(seen) / len(seen)) if seen else None
    except Exception:
        return None


def make_plan(torch, tao, ops, args):
    images = {}
    return [PlannedOp(tao, torch, op, images, use_split=not args.fp32_only, use_fused=not args.no_fused_check,
                      prepared=not args.no_prepared_weights) for op in ops]


def timed_passes(torch, plan, steps, warmup):
    """`warmup` untimed passes of the plan, then `steps` timed ones (per-operator HIP events inside)."""
    for _ in range(warmup):
        for p in plan:
            p.run(torch, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for p in plan:
            p.run(torch, True)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def graph_replay_ms(torch, tao, plan, steps):
    """One pass of the plan captured into a HIP graph (the entry points only enqueue kernels) and replayed:
    (ms per replay, violations seen by the last replay).  For the small configurations, whose pass is a few
    dozen launches of 4 - 80 us, this takes the launch spacing of the eager loop out."""
    for p in plan:
        p.run(torch, False)                                   # every cached scratch buffer exists before the capture
    torch.cuda.synchronize()
    gph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gph):
        for p in plan:
            p.run(torch, False)
    for _ in range(3):
        gph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        gph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    return ms, sum(tao.read_profile(p.prof)["violations"] for p in plan)


def plan_summary(tao, plan, ms_per_pass, what):
    """Whole-pass figures of one configuration: throughput, the matmul bound against the FP32 MFMA peak
    (algorithmic flop) and the streaming operators against the HBM peak (algorithmic bytes)."""
    elems = sum(p.n for p in plan)
    lin = [p for p in plan if p.kind == "linear"]
    out = {"workload": what, "operators": len(plan), "elements": elems, "ms_per_pass": ms_per_pass,
           "GB/s_verified": elems * 4 / (ms_per_pass * 1e-3) / 1e9,
           "violations": sum(tao.read_profile(p.prof)["violations"] for p in plan)}
    if lin:
        ms = sum(sum(_ms(p.bound_events)) for p in lin)
        fl = sum(p.flops * len(p.bound_events) for p in lin)
        out["matmul"] = {"TFLOP/s": fl / (ms * 1e-3) / 1e12, "frac_fp32_mfma_peak": fl / (ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
                         "ms_per_pass": ms / len(lin[0].bound_events),
                         "per_op": {p.name: {"shape": list(p.op.args["A"].shape) + [p.op.y_ref.shape[-1]], "path": p.path,
                                             "TFLOP/s": p.flops / (sum(_ms(p.bound_events)) / len(p.bound_events) * 1e-3) / 1e12,
                                             "ms": sum(_ms(p.bound_events)) / len(p.bound_events)} for p in lin}}
    st = [p for p in plan if p.kind != "linear"]
    if st:
        # streaming operators: bound (+ check in the same pass where fused); separate checks counted apart
        ms = sum(sum(_ms(p.bound_events)) for p in st)
        by = sum((_FUSED_BYTES if p.fused else _STREAM_BYTES)[p.kind] * p.n * len(p.bound_events) for p in st)
        out["streaming"] = {"GB/s": by / (ms * 1e-3) / 1e9, "frac_hbm": by / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                            "ms_per_pass": ms / len(st[0].bound_events)}
    chk = [p for p in plan if p.check_events]
    if chk:
        ms = sum(sum(_ms(p.check_events)) for p in chk)
        by = sum(12.0 * p.n * len(p.check_events) for p in chk)
        out["separate_checks"] = {"GB/s": by / (ms * 1e-3) / 1e9, "frac_hbm": by / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                  "ms_per_pass": ms / len(chk[0].check_events)}
    return out


def stream_bound_kernels(torch, tao, tao_inputs, dev):
    """The bound kernels that store tau (no check in the same pass) at 100 M elements and more:
    algorithmic bytes per second against the HBM peak."""
    out = {}
    g = torch.Generator(device=dev); g.manual_seed(777)

    def put(name, nbytes, fn, reps=5):
        ms = _event_time(torch, fn, reps, 1)
        out[name] = {"ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9, "frac_hbm": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}

    rows, cols = 65536, 2048                                          # 134 M elements, dense rows
    x = torch.randn((rows, cols), generator=g, device=dev) * 3
    y = torch.softmax(x, dim=-1); tau = torch.empty_like(x)
    put("bound_softmax_134M", 12.0 * x.numel(), lambda: tao.tao_bound_softmax(x, y, out=tau))
    rowpos = torch.arange(rows, device=dev) % cols
    x.masked_fill_(torch.arange(cols, device=dev)[None, :] > rowpos[:, None], float("-inf"))
    y = torch.softmax(x, dim=-1)
    put("bound_softmax_134M_causal", 12.0 * x.numel(), lambda: tao.tao_bound_softmax(x, y, out=tau))
    del x, y, tau
    rows, cols = 24576, 4096                                          # 100.7 M
    x = torch.randn((rows, cols), generator=g, device=dev)
    gam = 1 + 0.02 * torch.randn((cols,), generator=g, device=dev)
    y = tao_inputs.rmsnorm_f32(x, gam, 1e-6); tau = torch.empty_like(x)
    put("bound_rmsnorm_100M", 12.0 * x.numel(), lambda: tao.tao_bound_norm(1, x, y, gam, None, eps=1e-6, out=tau))
    t1 = torch.empty((rows,), device=dev)
    put("bound_sum_100M", 4.0 * x.numel(), lambda: tao.tao_bound_norm(3, x, None, out=t1))
    ym = x.sum(-1) / cols
    put("bound_mean_100M", 4.0 * x.numel(), lambda: tao.tao_bound_norm(4, x, ym, out=t1))
    flat_x, flat_y, flat_t = x.view(-1), y.view(-1), tau.view(-1)
    for nm, kind, nb in (("gelu", 0, 12.0), ("silu", 1, 8.0), ("mul", 2, 8.0)):
        put("bound_%s_100M" % nm, nb * flat_x.numel(), lambda kind=kind: tao.tao_bound_act(kind, flat_x, flat_y, out=flat_t))
    del x, y, tau, gam, flat_x, flat_y, flat_t
    rows, cols = 131072, 768                                          # 100.7 M
    x = torch.randn((rows, cols), generator=g, device=dev)
    gam = 1 + 0.02 * torch.randn((cols,), generator=g, device=dev); bet = 0.02 * torch.randn((cols,), generator=g, device=dev)
    y = tao_inputs.layernorm_f32(x, gam, bet, 1e-12); tau = torch.empty_like(x)
    put("bound_layernorm_100M", 12.0 * x.numel(), lambda: tao.tao_bound_norm(0, x, y, gam, bet, eps=1e-12, out=tau))
    put("bound_bn_affine_100M", 12.0 * x.numel(), lambda: tao.tao_bound_norm(2, x, y, gam, bet, out=tau))
    del x, y, tau
    return out


def projection_only(torch, tao, tao_inputs, dev, n, steps, warmup):
    """The two projections on n deviations claimed - ref of the check generator; thresholds: the
    deviations' own percentile profile (part of the elements is capped)."""
    claimed, ref, tau = tao_inputs.check_triplet(dev, n=n)
    delta = claimed - ref
    eprof = tao.tao_profile_errors(claimed, ref)
    del claimed, ref
    thr = torch.from_numpy(eprof["abs_p"].astype("float32")).to(dev)
    ws = torch.empty(tao.tao_project_workspace_bytes(n), dtype=torch.uint8, device=dev)
    out = torch.empty_like(delta)
    ms = _event_time(torch, lambda: tao.tao_project_empirical(delta, thr, 1.0, out=out, ws=ws), steps, warmup)
    capped = float((out != delta).float().mean().item())
    ms_clip = _event_time(torch, lambda: tao.tao_project_clip(delta, tau, 1.0, out=out), steps, warmup)
    return {"workload": "projections of Sec. 4.4, %d elements" % n,
            "project_empirical": {"ms": ms, "Gelem/s": n / (ms * 1e-3) / 1e9, "capped_frac": capped,
                                  "GB/s_at_72B_per_element": 72.0 * n / (ms * 1e-3) / 1e9},
            "project_clip": {"ms": ms_clip, "GB/s": 12.0 * n / (ms_clip * 1e-3) / 1e9,
                             "frac_hbm": 12.0 * n / (ms_clip * 1e-3) / 1e9 / PEAK_HBM_GBS}}


def cpu_baseline(ops, rows_per_op):
    """The oracle, as it stands, on the first `rows_per_op` output rows of every operator."""
    import numpy as np
    import oracle
    import tao_inputs
    from opmap import oracle_tau
    sample = []
    for op in ops:
        y = op.y_ref
        lead = y.shape[0] if y.dim() > 1 else 1
        if op.kind == "linear":
            A = op.args["A"]
            if A.dim() == 3:          # batched: take rows of the first batch entry
                args = {"A": A[0, :rows_per_op], "W": op.args["W"][0], "bias": None}
                sub = tao_inputs.Op(op.name, op.kind, args, y[0, :rows_per_op], op.claimed[0, :rows_per_op], op.attrs)
            else:
                args = {"A": A[:rows_per_op], "W": op.args["W"], "bias": op.args.get("bias")}
                sub = tao_inputs.Op(op.name, op.kind, args, y[:rows_per_op], op.claimed[:rows_per_op], op.attrs)
        else:
            def cut(t):
                if t is None or t.dim() == 1 and t.shape[0] != lead:
                    return t
                return t.reshape(-1, t.shape[-1])[:rows_per_op] if t.dim() > 1 else t
            args = {k: (cut(v) if k in ("x", "x2") else v) for k, v in op.args.items()}
            # (the first rows of a rotary operator are the first tokens: same table rows)
            sub = tao_inputs.Op(op.name, op.kind, args, cut(y), cut(op.claimed), op.attrs)
        # move to host before timing: the baseline is CPU work only
        sub.args = {k: (None if v is None else v.detach().cpu().contiguous()) for k, v in sub.args.items()}
        sub.y_ref = sub.y_ref.detach().cpu().contiguous()
        sub.claimed = sub.claimed.detach().cpu().contiguous()
        sample.append(sub)
    oracle.lib()
    t0 = time.perf_counter()
    elems = 0
    for sub in sample:
        tau = oracle_tau(oracle, sub)
        oracle.check_and_profile(sub.claimed.numpy(), sub.y_ref.numpy(), tau)
        elems += sub.y_ref.numel()
    dt = time.perf_counter() - t0
    return {"value": elems * 4 / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "first %d output rows of each of the %d operators (%d elements, %.1f s)" %
                      (rows_per_op, len(sample), elems, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--scale", type=int, default=1, help="shrink the workload (1 = full size)")
    ap.add_argument("--cpu-rows", type=int, default=2048, help="output rows per operator for the CPU oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stress", action="store_true", help="skip the 8192^3 / 67M-element side measurements")
    ap.add_argument("--no-configs", action="store_true", help="skip configurations 1, 2 and 4 and the 100 M-element bound kernels")
    ap.add_argument("--fp32-only", action="store_true", help="matmul bounds on the FP32 matrix cores only (no BF16-split path)")
    ap.add_argument("--no-fused-check", action="store_true",
                    help="store every tau and run the streaming check after every bound (default: the BF16-split "
                         "matmul kernel and all streaming bound kernels check their bound in registers)")
    ap.add_argument("--no-prepared-weights", action="store_true",
                    help="split the weights again in every step (default: their images are prepared once)")
    ap.add_argument("--projection-elems", type=int, default=0,
                    help="only time the two projections of Sec. 4.4 on this many synthetic elements and exit "
                         "(side measurement; used for the committed kernel trace)")
    ap.add_argument("--only-config", type=int, default=0,
                    help="only time this configuration (1, 2 or 4) and exit (side measurement; used for the committed kernel traces)")
    ap.add_argument("--only-product", type=int, default=0,
                    help="only time the BF16-split product of an n x n x n problem on prepared operand images and exit "
                         "(side measurement; used for the committed counter summary)")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run three 1 GiB element-wise copy kernels (reference kernel for scaling FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); got --gpus %d" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2510_16028_amd as tao
    import tao_inputs
    tao.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU (no CPU fallback)"
    dev = "cuda"
    torch.cuda.set_device(0)

    if args.projection_elems > 0:
        print(json.dumps(projection_only(torch, tao, tao_inputs, dev, args.projection_elems, args.steps, args.warmup)))
        return

    if args.only_product > 0:
        n = args.only_product
        g, A, W = tao_inputs.config5_operands(dev, size=n)
        a_img, w_img = tao.tao_split_operand(A), tao.tao_split_operand(W)
        out = torch.empty((n, n), device=dev)
        ms = _event_time(torch, lambda: tao.tao_bound_linear_images(a_img, w_img, n, n, n, out=out), args.steps, args.warmup)
        tf = 2.0 * n ** 3 / (ms * 1e-3) / 1e12
        print(json.dumps({"workload": "BF16-split product %d^3 on prepared operand images" % n, "ms": ms, "TFLOP/s": tf,
                          "issued_frac_of_bf16_peak": 8.0 * tf / PEAK_BF16_MFMA_TFLOPS}))
        return

    other = {1: ("config 1: one 64x256 @ 256x128 linear and a 64x128 softmax", lambda: tao_inputs.config1(dev)),
             2: ("config 2: BERT-base-shaped encoder block, seq 512, hidden 768, 12 heads, FFN 3072", lambda: tao_inputs.config2(dev)),
             4: ("config 4: ResNet-50-like conv stage, batch 32, 56x56x256, 3x3 conv (K = 2304) + BatchNorm-affine",
                 lambda: tao_inputs.config4(dev))}

    def measure_config(c):
        what, gen = other[c]
        cops = gen()
        cplan = make_plan(torch, tao, cops, args)
        ms = timed_passes(torch, cplan, args.steps, args.warmup)
        res = plan_summary(tao, cplan, ms, what)
        if c in (1, 2):
            gms, gviol = graph_replay_ms(torch, tao, cplan, max(args.steps, 20))
            res["hip_graph_replay"] = {"ms_per_pass": gms, "GB/s_verified": res["elements"] * 4 / (gms * 1e-3) / 1e9, "violations": gviol}
        del cplan, cops
        torch.cuda.empty_cache()
        return res

    if args.only_config:
        print(json.dumps(measure_config(args.only_config)))
        return

    ops = tao_inputs.config3(dev, scale=args.scale)
    plan = make_plan(torch, tao, ops, args)
    torch.cuda.synchronize()
    ms_per_step = timed_passes(torch, plan, args.steps, args.warmup)

    elems = sum(p.n for p in plan)
    violations = sum(tao.read_profile(p.prof)["violations"] for p in plan)
    value = elems * 4 / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the MFMA bound, all its launches in the timed region
    lin = [p for p in plan if p.kind == "linear"]
    lin_ms = sum(sum(_ms(p.bound_events)) for p in lin)
    lin_launches = sum(len(p.bound_events) for p in lin)
    lin_flops = sum(p.flops * len(p.bound_events) for p in lin)
    achieved = lin_flops / (lin_ms * 1e-3) / 1e12
    # the matmul bound, both paths together: algorithmic flop (2MNK) per second against the FP32 MFMA
    # peak the metric names; a BF16-split launch issues 8 BF16 products per operand pair and includes
    # the pre-pass of its activation (and of its weight, unless that was prepared)
    sp = [p for p in lin if p.split]
    paths = {}
    for nm, sel, mult, peak in (("bf16_split", sp, 8.0, PEAK_BF16_MFMA_TFLOPS), ("fp32", [p for p in lin if not p.split], 1.0, PEAK_FP32_MFMA_TFLOPS)):
        if sel:
            ms = sum(sum(_ms(p.bound_events)) for p in sel)
            fl = sum(p.flops * len(p.bound_events) for p in sel)
            paths[nm] = {"ops": [p.name for p in sel], "TFLOP/s": fl / (ms * 1e-3) / 1e12,
                         "issued_TFLOP/s": mult * fl / (ms * 1e-3) / 1e12, "issued_frac_of_own_peak": mult * fl / (ms * 1e-3) / 1e12 / peak}
    roofline = {"bound": "mfma", "kernel": "absgemm_split + absgemm_bound" if sp else "absgemm_bound",
                # operators checked in the matrix kernel's epilogue (tao_bound_check_linear): their launches, and
                # so this figure, contain the check
                "check_in_epilogue": [p.name for p in lin if p.fused],
                "prepared_weight_images": [p.name for p in lin if p.prepared],
                "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                # the two paths against the peak of the matrix cores each of them runs on: the FP32 path's
                # algorithmic flop against the FP32 MFMA peak, the BF16-split path's issued flop (8 BF16
                # products per operand pair) against the BF16 MFMA peak
                "frac_fp32_path_of_fp32_peak": paths["fp32"]["issued_frac_of_own_peak"] if "fp32" in paths else None,
                "frac_bf16_path_of_bf16_peak": paths["bf16_split"]["issued_frac_of_own_peak"] if "bf16_split" in paths else None,
                "paths": paths,
                # not measured by this run: the figure of the committed rocprofv3 --pmc summary of this command
                "traffic": measured_traffic("absgemm" if sp else "absgemm_bound") if args.scale == 1 else None,
                "traffic_source": "offline: profiles/bench_c3_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command)",
                "compulsory_bytes_per_launch": sum(p.min_bytes for p in lin) / len(lin),
                "launches": lin_launches, "avg_launch_ms": lin_ms / lin_launches,
                "flop_per_launch": lin_flops / lin_launches,
                "share_of_step": lin_ms / args.steps / ms_per_step}

    kernels = {}
    chk_ms = sum(sum(_ms(p.check_events)) for p in plan)
    chk_bytes = sum(12.0 * p.n * len(p.check_events) for p in plan)
    if chk_ms > 0:
        kernels["check_and_profile"] = {"GB/s": chk_bytes / (chk_ms * 1e-3) / 1e9,
                                        "frac_hbm": chk_bytes / (chk_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                        "avg_launch_ms": chk_ms / sum(len(p.check_events) for p in plan)}
    for kind in sorted({p.kind for p in plan if p.kind != "linear"}):
        for fused in (False, True):
            sel = [p for p in plan if p.kind == kind and p.fused == fused]
            if not sel:
                continue
            ms = sum(sum(_ms(p.bound_events)) for p in sel)
            by = sum((_FUSED_BYTES if fused else _STREAM_BYTES)[kind] * p.n * len(p.bound_events) for p in sel)
            kernels[("bound_check_" if fused else "bound_") + kind] = {
                "GB/s": by / (ms * 1e-3) / 1e9, "frac_hbm": by / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "avg_launch_ms": ms / sum(len(p.bound_events) for p in sel)}
    for p in lin:
        ms = sum(_ms(p.bound_events)) / len(p.bound_events)
        kernels["linear_" + p.name] = {"shape": list(p.op.args["A"].shape) + [p.op.y_ref.shape[-1]], "path": p.path,
                                       "TFLOP/s": p.flops / (ms * 1e-3) / 1e12, "ms": ms}

    configs = {}
    if not args.no_stress:
        # side measurements on the stress shapes (not part of `value`)
        g, A, W = tao_inputs.config5_operands(dev, size=8192)
        out = torch.empty((8192, 8192), device=dev)
        for flags, nm in ((0, "linear_8192^3"), (tao.FLAG_FAST_ACCUM, "linear_8192^3_fast_accum")):
            md = tao.FpModel(flags=flags)
            ms = _event_time(torch, lambda: tao.tao_bound_linear(A, W, model=md, out=out), 5, 1)
            tf = 2.0 * 8192 ** 3 / (ms * 1e-3) / 1e12
            kernels[nm] = {"ms": ms, "TFLOP/s": tf, "frac_mfma": tf / PEAK_FP32_MFMA_TFLOPS}
        ws5 = torch.empty(tao.tao_linear_split_workspace_bytes(8192, 8192, 8192, 1, True), dtype=torch.uint8, device=dev)
        ms = _event_time(torch, lambda: tao.tao_bound_linear_split(A, W, out=out, ws=ws5), 5, 1)
        tf = 2.0 * 8192 ** 3 / (ms * 1e-3) / 1e12
        kernels["linear_8192^3_bf16_split"] = {"ms": ms, "TFLOP/s": tf, "frac_mfma": tf / PEAK_FP32_MFMA_TFLOPS,
                                               "issued_frac_of_bf16_peak": 8.0 * tf / PEAK_BF16_MFMA_TFLOPS}
        a_img, w_img = tao.tao_split_operand(A), tao.tao_split_operand(W)
        ms = _event_time(torch, lambda: tao.tao_bound_linear_images(a_img, w_img, 8192, 8192, 8192, out=out), 5, 1)
        tf = 2.0 * 8192 ** 3 / (ms * 1e-3) / 1e12
        kernels["linear_8192^3_bf16_split_prepared_operands"] = {"ms": ms, "TFLOP/s": tf, "frac_mfma": tf / PEAK_FP32_MFMA_TFLOPS,
                                                                 "issued_frac_of_bf16_peak": 8.0 * tf / PEAK_BF16_MFMA_TFLOPS}
        # the clock the chip holds under either path's kernel (the peaks assume 2400 MHz)
        mhz = shader_clock_under(torch, lambda: tao.tao_bound_linear_images(a_img, w_img, 8192, 8192, 8192, out=out))
        kernels["linear_8192^3_bf16_split_prepared_operands"]["sclk_mhz"] = mhz
        if mhz:
            kernels["linear_8192^3_bf16_split_prepared_operands"]["issued_frac_of_bf16_peak_at_that_clock"] = \
                8.0 * tf / (PEAK_BF16_MFMA_TFLOPS * mhz / 2400.0)
        kernels["linear_8192^3"]["sclk_mhz"] = shader_clock_under(torch, lambda: tao.tao_bound_linear(A, W, out=out))
        del ws5, a_img, w_img
        tao.tao_bound_linear(A, W, out=out)      # the stored bound of the check below: the FP32 path's
        ref = A @ W.t()
        claimed, cls = tao_inputs.config5_claimed(g, ref, out)
        buf = tao.new_profile_buffer(ref.device)
        ms = _event_time(torch, lambda: tao.tao_check_and_profile(claimed, ref, out, out=buf, readback=False), 20, 2)
        prof = tao.read_profile(buf)
        kernels["check_67M"] = {"ms": ms, "GB/s": 12.0 * ref.numel() / (ms * 1e-3) / 1e9,
                                "frac_hbm": 12.0 * ref.numel() / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                "violations": prof["violations"], "expected_violations": int((cls == 2).sum()),
                                "p50": prof["p50"], "p99": prof["p99"], "p999": prof["p999"], "max_rel": prof["max_rel"]}
        # configuration 5 as one pass: the bound of the 8192^3 product checked on the spot against the
        # perturbed claims (the library's route: BF16-split kernel, check in its epilogue)
        ws5 = torch.empty(tao.tao_bound_check_linear_workspace_bytes(8192, 8192, 8192, 1, True), dtype=torch.uint8, device=dev)
        ms = _event_time(torch, lambda: tao.tao_bound_check_linear(A, W, None, ref, claimed, out=buf, ws=ws5, readback=False), 5, 1)
        prof = tao.read_profile(buf)
        tf = 2.0 * 8192 ** 3 / (ms * 1e-3) / 1e12
        configs["5"] = {"workload": "config 5: 8192^3 GEMM, U(-1,1) with 1 % x100, claims at 0.5 / 0.99 / 1.01 of the bound: bound + check of 67 M elements in one call",
                        "operators": 1, "elements": ref.numel(), "ms_per_pass": ms, "GB/s_verified": 4.0 * ref.numel() / (ms * 1e-3) / 1e9,
                        "violations": prof["violations"], "expected_violations": int((cls == 2).sum()),
                        "matmul": {"TFLOP/s": tf, "frac_fp32_mfma_peak": tf / PEAK_FP32_MFMA_TFLOPS,
                                   "issued_frac_of_bf16_peak": 8.0 * tf / PEAK_BF16_MFMA_TFLOPS, "path": "bf16_split+check"}}
        del ws5
        # the two projections of Sec. 4.4 on the 67M deviations claimed - ref; thresholds: the
        # deviations' own percentile profile (bin upper edges: part of the elements is capped) and a
        # third of it (every element is capped: the worst case of the last pass's random writes)
        delta = claimed - ref
        eprof = tao.tao_profile_errors(claimed, ref)
        pws = torch.empty(tao.tao_project_workspace_bytes(delta.numel()), dtype=torch.uint8, device=dev)
        pout = torch.empty_like(delta)
        for nm, f in (("project_empirical_67M", 1.0), ("project_empirical_67M_all_capped", 1.0 / 3)):
            thr = torch.from_numpy((eprof["abs_p"] * f).astype("float32")).to(dev)
            ms = _event_time(torch, lambda: tao.tao_project_empirical(delta, thr, 1.0, out=pout, ws=pws), 5, 1)
            kernels[nm] = {"ms": ms, "Gelem/s": delta.numel() / (ms * 1e-3) / 1e9,
                           "capped_frac": float((pout != delta).float().mean().item()),
                           "GB/s_at_72B_per_element": 72.0 * delta.numel() / (ms * 1e-3) / 1e9}
        ms = _event_time(torch, lambda: tao.tao_project_clip(delta, out, 1.0, out=pout), 20, 2)
        kernels["project_clip_67M"] = {"ms": ms, "GB/s": 12.0 * delta.numel() / (ms * 1e-3) / 1e9,
                                       "frac_hbm": 12.0 * delta.numel() / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
        ews = torch.empty(tao.tao_profile_workspace_bytes(delta.numel()), dtype=torch.uint8, device=dev)
        ebuf = torch.empty(ctypes_sizeof_error_profile(tao), dtype=torch.uint8, device=dev)
        ms = _event_time(torch, lambda: tao.tao_profile_errors(claimed, ref, out=ebuf, ws=ews, readback=False), 10, 2)
        kernels["profile_errors_67M"] = {"ms": ms, "GB/s": 8.0 * delta.numel() / (ms * 1e-3) / 1e9,
                                         "frac_hbm": 8.0 * delta.numel() / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
        del A, W, out, ref, claimed, cls, delta, pws, pout, ews, ebuf
        torch.cuda.empty_cache()

    if not args.no_configs and args.scale == 1:
        for c in (1, 2, 4):
            configs[str(c)] = measure_config(c)
        kernels.update(stream_bound_kernels(torch, tao, tao_inputs, dev))

    if args.copy_calib:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)       # an element-wise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    configs["3"] = plan_summary(tao, plan, ms_per_step, "config 3 (the workload of `value`)")
    configs["3"].pop("matmul", None); configs["3"].pop("streaming", None)      # detailed in `roofline` and `kernels`
    result = {
        "metric": "traced-operator GB/s verified (bound+check) & % FP32 MFMA/HBM peak, 1 GPU",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16 x 3 exact split / f32 (MFMA) + f64 (accumulation, scalars, check)" if sp
                  else "f32 (MFMA) + f64 (accumulation, scalars, check)"), "data": "synthetic",
        "config": {"workload": "config 3: Qwen3-8B-shaped decoder layer ops, FP32, seq %d: %d traced operators, "
                               "%d output elements verified per step" % (ops[0].y_ref.shape[0], len(plan), elems),
                   "scale": args.scale},
        "violations": violations,
        "roofline": roofline,
        "kernels": kernels,
        "configs": configs,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(ops, args.cpu_rows)
    print(json.dumps(result))


def ctypes_sizeof_error_profile(tao):
    import ctypes
    return ctypes.sizeof(tao.ErrorProfile)


if __name__ == "__main__":
    main()
