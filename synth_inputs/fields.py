"""Seeded Q/K/V fields and route vectors.

Recipe (per tensor in {Q,K,V}, per head, per channel): white N(0,1) noise on
the (F,H,W) grid, separable Gaussian blur (sigma = 2 tokens, taps out to
4 sigma, reflected boundary that repeats the edge sample), standardised to zero
mean / unit variance over the head, plus 0.5 * N(0,1) white noise, divided by
sqrt(1.25) so the result has unit variance.  Text tokens are plain N(0,1).
The values are rounded once to the layer's dtype; every consumer reads those
rounded bits.  The spatially smooth component gives neighbouring tokens
correlated keys, as video latents have; the white component keeps buckets
from being degenerate.
"""
import math
from typing import Tuple

import torch

from .configs import LayerConfig

_SIGMA = 2.0
_RADIUS = 8                       # 4 sigma
_NOISE = 0.5


def blur_matrix(n: int, sigma: float = _SIGMA, radius: int = _RADIUS) -> torch.Tensor:
    """Dense n x n matrix of a normalised Gaussian blur along one axis.

    Out-of-range taps fold back with the half-sample-symmetric reflection
    (d c b a | a b c d | d c b a), applied as often as needed, so short axes
    work too.
    """
    k = torch.arange(-radius, radius + 1, dtype=torch.float64)
    taps = torch.exp(-0.5 * (k / sigma) ** 2)
    taps = taps / taps.sum()
    m = torch.zeros(n, n, dtype=torch.float64)
    for i in range(n):
        for t, g in zip(range(-radius, radius + 1), taps.tolist()):
            p = (i + t) % (2 * n)
            if p >= n:
                p = 2 * n - 1 - p
            m[i, p] += g
    return m


def _head_seed(seed: int, tensor_id: int, head: int) -> int:
    return (seed * 1_000_003 + tensor_id * 10_007 + head * 101 + 17) & 0x7FFFFFFF


def _torch_dtype(name: str) -> torch.dtype:
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[name]


def make_head(cfg: LayerConfig, tensor_id: int, head: int, device="cpu") -> torch.Tensor:
    """One head of one tensor: [n_tokens, head_dim] in cfg.dtype (video tokens
    in frame-major raster order, then the text tokens)."""
    f, h, w = cfg.grid
    d = cfg.head_dim
    gen = torch.Generator(device=device)
    gen.manual_seed(_head_seed(cfg.seed, tensor_id, head))
    x = torch.randn(f, h, w, d, generator=gen, device=device, dtype=torch.float32)
    bf = blur_matrix(f).to(device=device, dtype=torch.float32)
    bh = blur_matrix(h).to(device=device, dtype=torch.float32)
    bw = blur_matrix(w).to(device=device, dtype=torch.float32)
    x = torch.einsum("af,fhwd->ahwd", bf, x)
    x = torch.einsum("bh,ahwd->abwd", bh, x)
    x = torch.einsum("cw,abwd->abcd", bw, x)
    x = (x - x.mean()) / x.std(unbiased=False)
    x = x + _NOISE * torch.randn(f, h, w, d, generator=gen, device=device, dtype=torch.float32)
    x = x / math.sqrt(1.0 + _NOISE * _NOISE)
    x = x.reshape(f * h * w, d)
    if cfg.n_text:
        t = torch.randn(cfg.n_text, d, generator=gen, device=device, dtype=torch.float32)
        x = torch.cat([x, t], dim=0)
    return x.to(_torch_dtype(cfg.dtype))


def make_qkv(cfg: LayerConfig, device="cpu", layout: int = 1
             ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Q, K, V of one layer.  layout 1: [heads, N, d]; layout 0: [N, heads, d]
    (both contiguous)."""
    out = []
    for tensor_id in range(3):
        buf = torch.empty(cfg.heads, cfg.n_tokens, cfg.head_dim,
                          dtype=_torch_dtype(cfg.dtype), device=device)
        for head in range(cfg.heads):
            buf[head] = make_head(cfg, tensor_id, head, device)
        if layout == 0:
            buf = buf.transpose(0, 1).contiguous()
        out.append(buf)
    return tuple(out)


def make_routes(cfg: LayerConfig) -> torch.Tensor:
    """uint8[heads] route vector.  Fixed order if the config gives one;
    otherwise head counts by largest-remainder rounding of the config's
    fractions, then a seeded shuffle over heads."""
    if cfg.fixed_routes is not None:
        return torch.tensor(cfg.fixed_routes, dtype=torch.uint8)
    if cfg.route_fractions is None:
        raise ValueError(f"config {cfg.name} has no route recipe; pass routes explicitly")
    exact = [fr * cfg.heads for fr in cfg.route_fractions]
    counts = [int(math.floor(e + 1e-9)) for e in exact]
    order = sorted(range(3), key=lambda r: -(exact[r] - counts[r]))
    for r in order[: cfg.heads - sum(counts)]:
        counts[r] += 1
    routes = torch.cat([torch.full((c,), r, dtype=torch.uint8) for r, c in enumerate(counts)])
    gen = torch.Generator(device="cpu")
    gen.manual_seed(_head_seed(cfg.seed, 7, 0))
    return routes[torch.randperm(cfg.heads, generator=gen)]
