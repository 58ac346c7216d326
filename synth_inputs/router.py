"""Seeded inputs of the attention router: timestep embeddings of a sampling schedule and one
d_t x 3 projection per head.

Only inputs are drawn here (nothing of the method's arithmetic: no softmax, no selection).  The
embedding is the usual sinusoidal code of the diffusion timestep; the projections are white noise
plus a planted trend along the direction in which the embedding moves over the schedule, so that,
as the paper observes for trained routers (section 4.3, "Attention patterns in VDiTs"), early
(noisy) steps lean towards the core-set branch and late steps towards the sliding-tile branch,
with a per-head offset that makes heads switch at different steps and leaves some on full
attention.
"""
import math
from typing import Tuple

import torch


def timestep_embedding(timesteps: torch.Tensor, d_t: int = 256, max_period: float = 10000.0) -> torch.Tensor:
    """[n_steps] -> [n_steps, d_t] float32: cos and sin of t at d_t / 2 geometrically spaced rates."""
    half = d_t // 2
    rates = torch.exp(-math.log(max_period) * torch.arange(half, dtype=torch.float64) / half)
    args = timesteps.to(torch.float64)[:, None] * rates[None, :]
    emb = torch.cat([torch.cos(args), torch.sin(args)], dim=1)
    if d_t % 2:
        emb = torch.cat([emb, torch.zeros(len(timesteps), 1, dtype=torch.float64)], dim=1)
    return emb.to(torch.float32)


def make_router_inputs(heads: int, n_steps: int = 10, d_t: int = 256, seed: int = 0,
                       trend: float = 6.0) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Returns (timesteps [n_steps], t_emb [n_steps, d_t] float32, w_r [heads, d_t, 3] float32),
    all on the CPU.  Timesteps run from 999 (pure noise, first sampling step) down to 0."""
    gen = torch.Generator(device="cpu").manual_seed(977 * seed + 13)
    timesteps = torch.linspace(999.0, 0.0, n_steps, dtype=torch.float64).round()
    t_emb = timestep_embedding(timesteps, d_t)
    w = 0.02 * torch.randn(heads, d_t, 3, generator=gen, dtype=torch.float64)
    # direction along which the embedding moves from the first to the last step
    u = (t_emb[0] - t_emb[-1]).to(torch.float64)
    mid = 0.5 * (t_emb[0] + t_emb[-1]).to(torch.float64)
    u = u / (u @ u)
    # core-set logit rises with <T, u> (early steps), sliding-tile logit falls; the per-head
    # offset moves the step at which the two cross, a per-head bias lifts full attention
    offset = torch.rand(heads, generator=gen, dtype=torch.float64) - 0.5
    w[:, :, 2] += trend * u[None, :]
    w[:, :, 1] -= trend * u[None, :]
    shift = (trend * offset)[:, None] * (mid / (mid @ mid))[None, :]
    w[:, :, 2] += shift
    w[:, :, 1] -= shift
    full_bias = 2.0 * torch.rand(heads, generator=gen, dtype=torch.float64) - 1.0
    w[:, :, 0] += full_bias[:, None] * (mid / (mid @ mid))[None, :]
    return timesteps, t_emb, w.to(torch.float32)
