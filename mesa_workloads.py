"""Seeded synthetic saved-activation sets shaped like the paper's ViT workloads.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds none of the method's arithmetic (no quantizer, no
dequantizer, no running-estimate update, no layer gradient): it only draws the
tensors a Transformer block would hand to the method -- attention maps, GELU
inputs, LayerNorm / Linear inputs, the forward's LayerNorm statistics, and
upstream gradients -- with torch's seeded generators, on whichever device the
caller names.  The same bits reach both sides because one side's tensors are
copied to the other; nothing is regenerated.

The shapes follow the five benchmark configurations (DeiT-Ti / DeiT-S / Swin-T
stage 1 / DeiT-B / long-sequence block, Sec. 5 of the paper for the model
families); the value distributions are stand-ins for ImageNet activations,
which are not available here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Sequence, Tuple

import torch


@dataclass(frozen=True)
class BlockSpec:
    name: str
    seed: int
    dtype: torch.dtype
    attn: Tuple[int, int, int, int]        # (B_or_windows, heads, rows, cols) of the attention map
    tokens: int                             # M = rows of the (M, D) token matrices
    dim: int                                # D
    mlp: int                                # hidden width of the MLP (GELU input is (M, mlp))
    heads: int                              # number of quantization groups of every tensor of the block
    sigma: Tuple[float, ...] = ()           # fixed per-head logit std; empty -> log-uniform in sigma_range
    sigma_range: Tuple[float, float] = (0.25, 4.0)
    ln_kind: str = "channel_mean"           # "channel_mean" | "outlier" | "channel_mean_std"
    outlier_scale: float = 20.0
    linears: Tuple[Tuple[int, int], ...] = ()   # (K, N_out) of the Linear layers whose dW is taken
    lam: float = 0.9

    @property
    def attn_layout(self):   # head-wise: (outer, groups, inner)
        b, h, r, c = self.attn
        return (b, h, r * c)

    @property
    def gelu_layout(self):   # channel groups over the MLP width
        return (self.tokens, self.heads, self.mlp // self.heads)

    @property
    def ln_layout(self):
        return (self.tokens, self.heads, self.dim // self.heads)


CONFIGS: Dict[int, BlockSpec] = {
    1: BlockSpec("deit_ti_block_b2", 0, torch.float32, (2, 3, 197, 197), 2 * 197, 192, 768, 3,
                 sigma=(0.5, 1.5, 4.0), ln_kind="channel_mean", linears=((192, 768),)),
    2: BlockSpec("deit_s_block_b128", 2, torch.float16, (128, 6, 197, 197), 128 * 197, 384, 1536, 6,
                 ln_kind="outlier", outlier_scale=20.0, linears=((384, 1536),)),
    3: BlockSpec("swin_t_stage1_b128", 3, torch.float16, (8192, 3, 49, 49), 128 * 3136, 96, 384, 3,
                 ln_kind="channel_mean_std"),
    4: BlockSpec("deit_b_block_b256", 4, torch.float16, (256, 12, 197, 197), 256 * 197, 768, 3072, 12,
                 ln_kind="outlier", outlier_scale=20.0,
                 linears=((768, 2304), (768, 768), (768, 3072), (3072, 768))),
    5: BlockSpec("long_seq_block_b8", 5, torch.float16, (8, 16, 4096, 4096), 8 * 4096, 1024, 4096, 16,
                 sigma_range=(0.25, 8.0), ln_kind="outlier", outlier_scale=50.0,
                 linears=((1024, 3072), (1024, 4096), (4096, 1024))),
}


def scaled(spec: BlockSpec, batch_div: int) -> BlockSpec:
    """The same block with the batch (leading) extent divided, for cases a CPU can check in full."""
    b, h, r, c = spec.attn
    return replace(spec, name=f"{spec.name}_div{batch_div}", attn=(max(1, b // batch_div), h, r, c),
                   tokens=max(1, spec.tokens // batch_div))


_TENSOR_IDS = {"attn": 1, "gelu": 2, "ln": 3, "lin": 4, "dy_attn": 5, "dy_gelu": 6, "dy_ln": 7, "dy_lin": 8,
               "gamma": 9, "sigma": 10, "chan": 11}


def _gen(spec: BlockSpec, what: str, draw: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(spec.seed * 1_000_003 + _TENSOR_IDS[what] * 1_009 + draw)
    return g


def head_sigmas(spec: BlockSpec) -> torch.Tensor:
    h = spec.attn[1]
    if spec.sigma:
        return torch.tensor(spec.sigma, dtype=torch.float32)
    g = _gen(spec, "sigma", 0, "cpu")
    lo, hi = spec.sigma_range
    u = torch.rand(h, generator=g, dtype=torch.float32)
    return torch.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))


def attention_map(spec: BlockSpec, draw: int = 0, device="cpu") -> torch.Tensor:
    """softmax(logits) with head h's logits ~ N(0, sigma_h^2); softmax in fp32, then cast."""
    b, h, r, c = spec.attn
    g = _gen(spec, "attn", draw, device)
    sig = head_sigmas(spec).to(device).view(1, h, 1, 1)
    out = torch.empty((b, h, r, c), dtype=spec.dtype, device=device)
    chunk = max(1, (1 << 26) // max(1, h * r * c))   # ~64M logits at a time
    for s in range(0, b, chunk):
        e = min(b, s + chunk)
        logits = torch.randn((e - s, h, r, c), generator=g, dtype=torch.float32, device=device) * sig
        out[s:e] = torch.softmax(logits, dim=-1).to(spec.dtype)
    return out


def gelu_input(spec: BlockSpec, draw: int = 0, device="cpu") -> torch.Tensor:
    g = _gen(spec, "gelu", draw, device)
    return _randn((spec.tokens, spec.mlp), g, spec.dtype, device)


def _randn(shape, g, dtype, device) -> torch.Tensor:
    out = torch.empty(shape, dtype=dtype, device=device)
    rows = shape[0]
    per = max(1, (1 << 26) // max(1, out[0].numel()))
    for s in range(0, rows, per):
        e = min(rows, s + per)
        out[s:e] = torch.randn((e - s,) + tuple(shape[1:]), generator=g, dtype=torch.float32, device=device).to(dtype)
    return out


def token_matrix(spec: BlockSpec, what: str = "ln", draw: int = 0, device="cpu", width: Optional[int] = None) -> torch.Tensor:
    """LayerNorm / Linear input of shape (tokens, width or dim)."""
    d = width or spec.dim
    g = _gen(spec, what, draw, device)
    x = torch.randn((spec.tokens, d), generator=g, dtype=torch.float32, device=device)
    if spec.ln_kind in ("channel_mean", "channel_mean_std"):
        gc = _gen(spec, "chan", draw if what == "ln" else 100 + draw, "cpu")
        mu = (torch.rand(d, generator=gc, dtype=torch.float32) * 4.0 - 2.0).to(device)
        if spec.ln_kind == "channel_mean_std":
            sd = (0.5 + 2.5 * torch.rand(d, generator=gc, dtype=torch.float32)).to(device)
            x = x * sd
        x = x + mu
    elif spec.ln_kind == "outlier":
        mask = torch.rand((spec.tokens, d), generator=g, dtype=torch.float32, device=device) < 1e-3
        x = torch.where(mask, x * spec.outlier_scale, x)
    else:
        raise ValueError(spec.ln_kind)
    return x.to(spec.dtype)


def layernorm_stats(x: torch.Tensor, eps: float = 1e-5):
    """What the exact forward keeps besides the input: per-row mean and 1/sqrt(var + eps), fp32."""
    xf = x.float()
    mean = xf.mean(dim=-1)
    var = xf.var(dim=-1, unbiased=False)
    return mean.contiguous(), torch.rsqrt(var + eps).contiguous()


def layernorm_gamma(spec: BlockSpec, device="cpu") -> torch.Tensor:
    g = _gen(spec, "gamma", 0, "cpu")
    return (0.5 + torch.rand(spec.dim, generator=g, dtype=torch.float32)).to(spec.dtype).to(device)


def upstream_grad(spec: BlockSpec, what: str, shape: Sequence[int], device="cpu", draw: int = 0) -> torch.Tensor:
    g = _gen(spec, what, draw, device)
    return _randn(tuple(shape), g, spec.dtype, device)


def small_case(dtype=torch.float32, seed=11, B=2, H=3, N=19, D=24, mlp=48) -> BlockSpec:
    """A tiny block with ragged extents for brute-force checks."""
    return BlockSpec(f"tiny_{N}_{D}", seed, dtype, (B, H, N, N), B * N, D, mlp, H,
                     sigma=tuple(0.5 * (k + 1) for k in range(H)), ln_kind="channel_mean", linears=((D, mlp),))
