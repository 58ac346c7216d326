"""Glue shared by the tests: config -> oracle spec, tensor -> fp64 array."""
import numpy as np
import torch

from oracle import vorta_oracle as vo
from synth_inputs import LayerConfig


def spec_of(cfg: LayerConfig, **over) -> vo.LayerSpec:
    kw = dict(grid=cfg.grid, tile=cfg.tile, window=cfg.window, bucket=cfg.bucket,
              keep_num=cfg.keep_num, keep_den=cfg.keep_den, n_text=cfg.n_text,
              rope_dims=cfg.rope_dims, rope_theta=cfg.rope_theta)
    kw.update(over)
    return vo.LayerSpec(**kw)


def f64(t) -> np.ndarray:
    """Widen a (possibly bf16, possibly device) tensor to an fp64 NumPy array."""
    if isinstance(t, torch.Tensor):
        return t.detach().to("cpu", torch.float64).numpy()
    return np.asarray(t, dtype=np.float64)


def smooth_field(rng, grid, d, noise=0.5):
    """A small correlated field for oracle tests (not the benchmark recipe):
    cumulative-sum smoothing keeps neighbours similar without any library."""
    F, H, W = grid
    x = rng.standard_normal((F, H, W, d))
    x = x + np.roll(x, 1, 0) + np.roll(x, 1, 1) + np.roll(x, 1, 2)
    x = x / x.std() + noise * rng.standard_normal((F, H, W, d))
    return x.reshape(F * H * W, d)
