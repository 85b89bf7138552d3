"""Seeded synthetic workloads for the tolerance engine.

This module only *makes inputs*: operator operands, the verifier's re-executed
FP32 outputs (y_ref) and the claimed outputs that are to be checked.  It holds
none of the method's arithmetic (no bound, no check, no histogram) and serves
both sides of every parity test: the same tensors go to the GPU library and,
as numpy arrays, to the CPU oracle.

Shapes and value distributions follow the five benchmark configurations: they
stand in for traces of CNN / Transformer / LLM inference; no dataset item and
no trained weight is used.  `scale` shrinks the sequence / batch dimension so
that the oracle finishes in seconds; scale=1 is the full size.

Tensors are produced with torch on the requested device (CPU for the small
parity cases, the GPU for full-size runs) from a torch.Generator seeded per
configuration; FP32 re-executions use plain torch FP32 operators.
"""
import math
from dataclasses import dataclass, field
from typing import Dict, Optional

import torch

SEED0 = 20251016


@dataclass
class Op:
    """One traced operator: what kind of bound it needs, its operands, the
    verifier's own output and the claimed output."""
    name: str
    kind: str                      # linear | softmax | layernorm | rmsnorm | bn_affine | gelu | silu | mul | add | sum | mean | rope
    args: Dict[str, Optional[torch.Tensor]]
    y_ref: torch.Tensor
    claimed: torch.Tensor
    attrs: Dict[str, object] = field(default_factory=dict)   # "weight": W is a committed model weight (constant across inputs)


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def randn(g, shape, std=1.0):
    return torch.randn(shape, generator=g, device=g.device, dtype=torch.float32) * std


def rand_uniform(g, shape, lo=-1.0, hi=1.0):
    return torch.rand(shape, generator=g, device=g.device, dtype=torch.float32) * (hi - lo) + lo


def heavy_tailed(g, shape, frac=0.01, factor=100.0):
    """U(-1,1) with a fraction of the entries multiplied by `factor`."""
    x = rand_uniform(g, shape)
    hit = torch.rand(shape, generator=g, device=g.device) < frac
    return torch.where(hit, x * factor, x)


def ulp_noise(g, y, max_ulps=3):
    """Move every element by k in {0..max_ulps} units in the last place, random sign
    (an integer step on the bit pattern, away from or toward zero)."""
    k = torch.randint(0, max_ulps + 1, y.shape, generator=g, device=g.device, dtype=torch.int32)
    s = torch.randint(0, 2, y.shape, generator=g, device=g.device, dtype=torch.int32) * 2 - 1
    bits = y.contiguous().view(torch.int32)
    # keep zero and the smallest magnitudes from crossing zero
    step = torch.where(bits.abs() > max_ulps, k * s, torch.zeros_like(k))
    return (bits + step).view(torch.float32)


def matmul_permuted_k(g, A, Wnk):
    """FP32 A @ Wnk^T with the reduction dimension visited in a seeded random order."""
    K = A.shape[-1]
    perm = torch.randperm(K, generator=g, device=g.device)
    return A[..., perm].contiguous() @ Wnk[..., perm].contiguous().transpose(-1, -2)


def matmul_split_k(A, Wnk, slabs):
    """FP32 A @ Wnk^T computed as `slabs` partial products over K that are then summed."""
    K = A.shape[-1]
    step = (K + slabs - 1) // slabs
    acc = None
    for k0 in range(0, K, step):
        part = A[..., k0:k0 + step] @ Wnk[..., k0:k0 + step].transpose(-1, -2)
        acc = part if acc is None else acc + part
    return acc


def softmax_f32(x):
    m = x.max(dim=-1, keepdim=True).values
    e = torch.exp(x - m)
    return e / e.sum(dim=-1, keepdim=True)


def softmax_f32_reordered(g, x):
    """Same algorithm with the row sum taken over a permuted column order."""
    n = x.shape[-1]
    perm = torch.randperm(n, generator=g, device=g.device)
    m = x.max(dim=-1, keepdim=True).values
    e = torch.exp(x - m)
    s = e[..., perm].contiguous().sum(dim=-1, keepdim=True)
    return e / s


def layernorm_f32(x, gamma, beta, eps, perm=None):
    xs = x if perm is None else x[..., perm].contiguous()
    n = x.shape[-1]
    mu = xs.sum(dim=-1, keepdim=True) / n
    d = x - mu
    ds = d if perm is None else d[..., perm].contiguous()
    var = (ds * ds).sum(dim=-1, keepdim=True) / n
    r = torch.rsqrt(var + torch.tensor(eps, dtype=torch.float32, device=x.device))
    return d * r * gamma + beta


def rmsnorm_f32(x, gamma, eps, perm=None):
    xs = x if perm is None else x[..., perm].contiguous()
    n = x.shape[-1]
    v = (xs * xs).sum(dim=-1, keepdim=True) / n
    r = torch.rsqrt(v + torch.tensor(eps, dtype=torch.float32, device=x.device))
    return gamma * (x * r)


def gelu_f32(x):
    return (0.5 * x) * (1.0 + torch.erf(x * torch.tensor(1.0 / math.sqrt(2.0), dtype=torch.float32, device=x.device)))


def silu_f32(x):
    return x / (1.0 + torch.exp(-x))


def gelu_via_f64(x):
    """An honest variant execution: the whole expression in binary64, rounded once."""
    xd = x.double()
    return (0.5 * xd * (1.0 + torch.erf(xd / math.sqrt(2.0)))).float()


def silu_via_f64(x):
    xd = x.double()
    return (xd / (1.0 + torch.exp(-xd))).float()


def affine_fused(x, s, t):
    """x*s + t with a single rounding (what a fused multiply-add kernel returns)."""
    return (x.double() * s.double() + t.double()).float()


def rope_tables(seq, hd, theta, device):
    """cos / sin tables [seq, hd/2] of the rotary embedding, binary32."""
    inv = theta ** (-torch.arange(0, hd, 2, device=device, dtype=torch.float32) / hd)
    ang = torch.arange(seq, device=device, dtype=torch.float32)[:, None] * inv[None, :]
    return torch.cos(ang), torch.sin(ang)


def rope_rows(x, cos, sin, heads):
    """Rotate-half embedding of x [seq*heads, hd] (token-major rows), binary32."""
    hd = x.shape[-1]
    xs = x.reshape(-1, heads, hd)
    c, s = cos[:, None, :], sin[:, None, :]
    a, b = xs[..., : hd // 2], xs[..., hd // 2:]
    return torch.cat([a * c - b * s, b * c + a * s], dim=-1).reshape(x.shape)


# ------------------------------------------------------------------ configurations

def config1(device="cpu", seed=SEED0 + 1):
    """Single FP32 linear 64x256 @ 256x128 (+ a 64x128 softmax); claimed = result +- {0..3} ulp."""
    g = _gen(seed, device)
    X = randn(g, (64, 256))
    Wkn = randn(g, (256, 128))                 # [K, N] layout: trans_w
    y = X @ Wkn
    ops = [Op("linear", "linear", {"A": X, "W": Wkn, "bias": None}, y, ulp_noise(g, y), {"trans_w": 1})]
    p = softmax_f32(y)
    ops.append(Op("softmax", "softmax", {"x": y}, p, softmax_f32_reordered(g, y)))
    return ops


def config2(device="cpu", seed=SEED0 + 2, scale=1):
    """BERT-base-shaped encoder block: seq 512/scale, hidden 768, 12 heads x 64, FFN 3072,
    weights and biases N(0, 0.02), activations N(0, 1), LayerNorm eps 1e-12, GELU(erf);
    claimed = recomputation with a permuted reduction order."""
    g = _gen(seed, device)
    S, H, NH, HD, F = max(512 // scale, 8), 768, 12, 64, 3072
    eps = 1e-12
    ops = []
    x = randn(g, (S, H))

    def linear(name, a, n_out):
        W = randn(g, (n_out, a.shape[-1]), 0.02)
        b = randn(g, (n_out,), 0.02)
        y = a @ W.t() + b
        ops.append(Op(name, "linear", {"A": a, "W": W, "bias": b}, y, matmul_permuted_k(g, a, W) + b, {"weight": True}))
        return y

    def layernorm(name, a):
        gam = 1.0 + randn(g, (H,), 0.02)
        bet = randn(g, (H,), 0.02)
        y = layernorm_f32(a, gam, bet, eps)
        perm = torch.randperm(H, generator=g, device=g.device)
        ops.append(Op(name, "layernorm", {"x": a, "gamma": gam, "beta": bet}, y,
                      layernorm_f32(a, gam, bet, eps, perm), {"eps": eps}))
        return y

    qkv = linear("qkv", x, 3 * H)
    q, k, v = [t.reshape(S, NH, HD).permute(1, 0, 2).contiguous() for t in qkv.split(H, dim=-1)]
    q = q * (1.0 / math.sqrt(HD))
    scores = q @ k.transpose(-1, -2)
    ops.append(Op("qk", "linear", {"A": q, "W": k, "bias": None}, scores, matmul_permuted_k(g, q, k)))
    p = softmax_f32(scores)
    ops.append(Op("softmax", "softmax", {"x": scores}, p, softmax_f32_reordered(g, scores)))
    ctx = p @ v
    vt = v.transpose(-1, -2).contiguous()
    ops.append(Op("pv", "linear", {"A": p, "W": v, "bias": None}, ctx, matmul_permuted_k(g, p, vt), {"trans_w": 1}))
    ctx2 = ctx.permute(1, 0, 2).reshape(S, H).contiguous()
    attn = linear("out_proj", ctx2, H)
    res1 = attn + x
    ops.append(Op("residual1", "add", {"x": attn, "x2": x}, res1, res1.clone()))   # IEEE add: bit-identical everywhere
    h1 = layernorm("ln1", res1)
    f1 = linear("ffn_up", h1, F)
    a1 = gelu_f32(f1)
    ops.append(Op("gelu", "gelu", {"x": f1}, a1, gelu_via_f64(f1)))
    f2 = linear("ffn_down", a1, H)
    res2 = f2 + h1
    ops.append(Op("residual2", "add", {"x": f2, "x2": h1}, res2, res2.clone()))
    layernorm("ln2", res2)
    return ops


def config3(device="cpu", seed=SEED0 + 3, scale=1):
    """Qwen3-8B-shaped decoder layer: hidden 4096, intermediate 12288, 32 q heads / 8 kv heads,
    head_dim 128, seq 2048/scale, RMSNorm eps 1e-6, SiLU-gated MLP, RoPE theta 1e6, causal
    softmax, weights N(0, 0.02); claimed = split-K recomputation."""
    g = _gen(seed, device)
    S, H, I, NQ, NKV, HD = max(2048 // scale, 16), 4096, 12288, 32, 8, 128
    if scale > 1:                               # keep the small case quick: shrink widths too
        H, I = 4096 // min(scale, 8), 12288 // min(scale, 8)
        NQ, NKV = max(32 // min(scale, 8), 4), max(8 // min(scale, 8), 1)
    eps, G = 1e-6, NQ // NKV
    slabs = [4, 8, 16]
    ops = []
    x = randn(g, (S, H))

    def linear(name, a, n_out, si):
        W = randn(g, (n_out, a.shape[-1]), 0.02)
        y = a @ W.t()
        ops.append(Op(name, "linear", {"A": a, "W": W, "bias": None}, y, matmul_split_k(a, W, slabs[si % 3]), {"weight": True}))
        return y

    def rmsnorm(name, a):
        gam = 1.0 + randn(g, (a.shape[-1],), 0.02)
        y = rmsnorm_f32(a, gam, eps)
        perm = torch.randperm(a.shape[-1], generator=g, device=g.device)
        ops.append(Op(name, "rmsnorm", {"x": a, "gamma": gam}, y, rmsnorm_f32(a, gam, eps, perm), {"eps": eps}))
        return y

    h = rmsnorm("input_norm", x)
    q = linear("q_proj", h, NQ * HD, 0)
    k = linear("k_proj", h, NKV * HD, 1)
    v = linear("v_proj", h, NKV * HD, 2).reshape(S, NKV, HD).permute(1, 0, 2).contiguous()
    cos, sin = rope_tables(S, HD, 1e6, device)

    def rotary(name, a, heads):
        rows = a.reshape(S * heads, HD)
        y = rope_rows(rows, cos, sin, heads)
        # two products and one addition leave no order to vary: the honest claim is bit-identical
        # (a fused variant or the correctly rounded rotation can differ from y by up to 1.5 tau,
        # which only a scale factor alpha = 2 admits)
        ops.append(Op(name, "rope", {"x": rows, "cos": cos, "sin": sin}, y, y.clone(), {"inner": heads}))
        return y.reshape(S, heads, HD).permute(1, 0, 2)

    q = rotary("q_rope", q, NQ) * (1.0 / math.sqrt(HD))
    k = rotary("k_rope", k, NKV).contiguous()
    # grouped-query attention: the G query heads of one kv head are stacked along M
    qg = q.reshape(NKV, G, S, HD).reshape(NKV, G * S, HD).contiguous()
    scores = qg @ k.transpose(-1, -2)                                   # [NKV, G*S, S]
    ops.append(Op("qk", "linear", {"A": qg, "W": k, "bias": None}, scores, matmul_split_k(qg, k, 4)))
    rowpos = torch.arange(G * S, device=device) % S
    mask = torch.arange(S, device=device)[None, :] > rowpos[:, None]    # above the diagonal
    masked = scores.masked_fill(mask[None], float("-inf"))
    p = softmax_f32(masked)
    ops.append(Op("softmax", "softmax", {"x": masked}, p, softmax_f32_reordered(g, masked)))
    ctx = p @ v
    vt = v.transpose(-1, -2).contiguous()
    ops.append(Op("pv", "linear", {"A": p, "W": v, "bias": None}, ctx, matmul_split_k(p, vt, 8), {"trans_w": 1}))
    ctx2 = ctx.reshape(NKV, G, S, HD).reshape(NQ, S, HD).permute(1, 0, 2).reshape(S, NQ * HD).contiguous()
    o = linear("o_proj", ctx2, H, 0)
    res1 = o + x
    ops.append(Op("residual1", "add", {"x": o, "x2": x}, res1, res1.clone()))
    h2 = rmsnorm("post_norm", res1)
    gate = linear("gate_proj", h2, I, 1)
    up = linear("up_proj", h2, I, 2)
    act = silu_f32(gate)
    ops.append(Op("silu", "silu", {"x": gate}, act, silu_via_f64(gate)))
    prod = act * up
    ops.append(Op("gate_mul", "mul", {"x": act, "x2": up}, prod, prod.clone()))
    down = linear("down_proj", prod, H, 0)
    res2 = down + res1
    ops.append(Op("residual2", "add", {"x": down, "x2": res1}, res2, res2.clone()))
    return ops


def config4(device="cpu", seed=SEED0 + 4, scale=1):
    """ResNet-50-like conv stage as an im2col GEMM: batch 32/scale, 56x56x256 half-normal input,
    3x3 conv to 256 channels, stride 1, pad 1 (K = 2304), He-normal weights, then a per-channel
    BatchNorm-affine; claimed = permuted-order recomputation."""
    g = _gen(seed, device)
    B, HW, C, CO = max(32 // scale, 1), (56 if scale == 1 else 12), 256, 256
    x = randn(g, (B, C, HW, HW)).abs()                                  # ReLU outputs: half-normal
    cols = torch.nn.functional.unfold(x, kernel_size=3, padding=1)       # [B, C*9, HW*HW]
    A = cols.transpose(1, 2).reshape(B * HW * HW, C * 9).contiguous()
    W = randn(g, (CO, C * 9), math.sqrt(2.0 / (C * 9)))
    y = A @ W.t()
    ops = [Op("conv_im2col", "linear", {"A": A, "W": W, "bias": None}, y, matmul_permuted_k(g, A, W), {"weight": True})]
    # the same convolution in the layout of the native entry point: channels-last input and
    # filters [Cout][R][S][C] (the patch matrix above orders its columns (c, r, s) instead)
    ops[0].attrs["conv"] = {"x": x.permute(0, 2, 3, 1).contiguous(),
                            "w": W.reshape(CO, C, 3, 3).permute(0, 2, 3, 1).contiguous(), "padding": 1}
    s = 1.0 + randn(g, (CO,), 0.1)
    t = randn(g, (CO,), 0.1)
    z = y * s + t
    # an unfused multiply-add is deterministic: the honest claim is bit-identical.  (A fused
    # variant differs from it by up to u|xs| + 2u|y|, which only a scale factor alpha = 2 admits.)
    ops.append(Op("bn_affine", "bn_affine", {"x": y, "scale": s, "shift": t}, z, z.clone()))
    return ops


def config5_operands(device="cpu", seed=SEED0 + 5, size=8192):
    """Stress GEMM operands: size^3, entries U(-1,1) with 1 % multiplied by 100."""
    g = _gen(seed, device)
    A = heavy_tailed(g, (size, size))
    W = heavy_tailed(g, (size, size))
    return g, A, W


def config5_claimed(g, ref, tau):
    """claimed = ref +- f*tau with f drawn per element from {0.5, 0.99, 1.01} (probabilities
    1/2, 1/4, 1/4) and a random sign; returns (claimed, f_class) with f_class in {0, 1, 2}.
    Arithmetic in binary64 so that the 1 % margins survive the final rounding to binary32."""
    cls = torch.randint(0, 4, ref.shape, generator=g, device=g.device)
    cls = torch.where(cls == 0, torch.zeros_like(cls), cls - 1)          # {0,0,1,2}
    f = torch.tensor([0.5, 0.99, 1.01], dtype=torch.float64, device=ref.device)[cls]
    sgn = torch.randint(0, 2, ref.shape, generator=g, device=g.device).double() * 2 - 1
    claimed = (ref.double() + sgn * f * tau.double()).float()
    return claimed, cls


def check_triplet(device="cpu", seed=SEED0 + 6, n=1 << 20):
    """(claimed, ref, tau) for exercising the check/profile pass alone: ref ~ N(0,1), relative
    deviations log-uniform over 1e-8..1e-3, tau a noisy multiple of |ref| so that a known-size
    fraction of elements violates."""
    g = _gen(seed, device)
    ref = randn(g, (n,))
    mag = 10.0 ** rand_uniform(g, (n,), -8.0, -3.0)
    claimed = ref * (1.0 + randn(g, (n,)) * mag)
    tau = ref.abs() * 10.0 ** rand_uniform(g, (n,), -7.0, -3.0)
    return claimed, ref, tau
