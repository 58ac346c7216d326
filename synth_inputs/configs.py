"""The five layer shapes the parity tests and the benchmark run on.

Shapes follow video-DiT attention layers (latent grid F x H x W flattened
frame-major into L tokens, paper section 2 "3D self-attention"); the sparse
branches use the paper's bucket (2,3,2) and core-set ratio 0.5 (appendix,
"Implementation details").  Route codes follow the gate order of Eq. 3:
0 = full, 1 = sliding tile window, 2 = core-set (long range).
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

ROUTE_FULL = 0
ROUTE_WINDOW = 1
ROUTE_CORESET = 2


@dataclass(frozen=True)
class LayerConfig:
    name: str
    grid: Tuple[int, int, int]            # latent (F, H, W)
    heads: int
    head_dim: int
    dtype: str                            # "fp32" | "bf16"
    tile: Tuple[int, int, int]            # tokens per tile
    window: Tuple[int, int, int]          # window, in tiles
    seed: int
    n_text: int = 0                       # tokens appended after the video tokens
    bucket: Tuple[int, int, int] = (2, 3, 2)
    keep_num: int = 1                     # core-set ratio r = keep_num / keep_den
    keep_den: int = 2
    route_fractions: Optional[Tuple[float, float, float]] = None   # (full, window, core-set)
    fixed_routes: Optional[Tuple[int, ...]] = None
    rope_dims: Optional[Tuple[int, int, int]] = None   # channels turned by the F, H, W position; None = no RoPE
    rope_theta: float = 10000.0

    @property
    def n_video(self) -> int:
        f, h, w = self.grid
        return f * h * w

    @property
    def n_tokens(self) -> int:
        return self.n_video + self.n_text


CONFIGS = (
    LayerConfig("tiny", (4, 8, 8), 2, 64, "fp32", (2, 4, 4), (3, 3, 3), seed=0,
                fixed_routes=None),       # every head is run under each of the 3 routes
    LayerConfig("single", (12, 16, 16), 8, 128, "bf16", (4, 4, 4), (3, 3, 3), seed=1,
                fixed_routes=(0, 0, 1, 1, 1, 2, 2, 2)),
    LayerConfig("wan480p", (21, 30, 52), 40, 128, "bf16", (3, 6, 4), (3, 3, 3), seed=2,
                route_fractions=(0.20, 0.40, 0.40)),
    LayerConfig("wan720p", (21, 45, 80), 40, 128, "bf16", (3, 5, 8), (3, 3, 3), seed=3,
                route_fractions=(0.15, 0.45, 0.40)),
    LayerConfig("hunyuan720p", (33, 45, 80), 24, 128, "bf16", (3, 5, 8), (3, 3, 3), seed=4,
                n_text=256, route_fractions=(0.10, 0.50, 0.40)),
)


# Not one of the five benchmark configs: the operating point the paper itself reports
# (appendix "Methodological details": HunyuanVideo at 720p / 117 frames = 30x45x80 latent grid,
# sliding window of (18, 27, 24) tokens = 3x3x3 tiles of (6, 9, 8), bucket (2, 3, 2), r = 1/2,
# full attention chosen for under 0.2 % of the heads -- here none of the 24).
EXTRA_CONFIGS = (
    LayerConfig("paper720p", (30, 45, 80), 24, 128, "bf16", (6, 9, 8), (3, 3, 3), seed=5,
                n_text=256, route_fractions=(0.0, 0.5, 0.5)),
    # the same appendix's second model: Wan 2.1 at 720p / 77 frames = 20x45x80 latents, 40 heads,
    # no text tokens in self-attention; 6 frames per tile do not divide 20, so the last tile
    # layer along F is clipped to 2 frames
    LayerConfig("paper_wan720p", (20, 45, 80), 40, 128, "bf16", (6, 9, 8), (3, 3, 3), seed=6,
                route_fractions=(0.0, 0.5, 0.5)),
)


def get_config(name: str) -> LayerConfig:
    for c in CONFIGS + EXTRA_CONFIGS:
        if c.name == name:
            return c
    raise KeyError(f"unknown config {name!r}; have {[c.name for c in CONFIGS]}")
