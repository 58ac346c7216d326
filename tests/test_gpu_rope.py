"""GPU parity with the rotary position embedding switched on: the row pass and the rotating pool
against the oracle's rotation, then whole layers under every route and the soft mixture."""
import numpy as np
import pytest
import torch

import paper_2505_18809_amd as vorta
from oracle import vorta_oracle as vo
from synth_inputs import LayerConfig, get_config, make_qkv
from helpers import f64, spec_of
from test_gpu_parity import check_layer, say, hnd, TOL, DEV

pytestmark = pytest.mark.gpu

WAN_ROPE = (44, 42, 42)        # a 128-channel head split the way Wan-style video DiTs split it
HUNYUAN_ROPE = (16, 56, 56)


def roped_cfg(name, grid, heads, dtype, tile, routes, d=128, n_text=0, seed=71, rope=WAN_ROPE, theta=10000.0, **kw):
    return LayerConfig(name, grid, heads, d, dtype, tile, (3, 3, 3), seed=seed, n_text=n_text,
                       fixed_routes=tuple(routes), rope_dims=rope, rope_theta=theta, **kw)


@pytest.mark.parametrize("layout", [1, 0])
@pytest.mark.parametrize("dtype,d,rope", [("bf16", 128, WAN_ROPE), ("bf16", 128, (0, 64, 60)), ("fp32", 64, (16, 24, 24)),
                                          ("fp32", 128, HUNYUAN_ROPE)])
def test_row_pass_and_rotating_pool_match_the_oracles_rotation(dtype, d, rope, layout):
    cfg = roped_cfg("rope_rows", (5, 7, 9), 4, dtype, (2, 3, 4), [0, 2, 1, 2], d=d, n_text=6, rope=rope, theta=256.0)
    say(f"rope rows {dtype} d={d} rope={rope} layout={layout}")
    q, k, v = make_qkv(cfg, DEV, layout)
    plan = vorta.plan_for(cfg, layout=layout)
    routes = np.array(cfg.fixed_routes, dtype=np.uint8)
    spec = spec_of(cfg)
    L = cfg.n_video
    dst = torch.full_like(q, 3.0)
    vorta.vorta_rope_apply(plan, q, routes, dst)
    torch.cuda.synchronize()
    qh, dh = hnd(q, layout), hnd(dst, layout)
    rel = 2.0 ** -8 if dtype == "bf16" else 1e-6
    for h, r in enumerate(routes):
        if r == 2:
            assert (dh[h] == 3.0).all()                        # route-2 heads rotate inside pool(): rows untouched
            continue
        want = vo.rope_video_rows(f64(qh[h]), spec)
        assert np.abs(f64(dh[h]) - want).max() <= rel * max(1.0, np.abs(want).max())
        assert torch.equal(dh[h][L:], qh[h][L:])               # text rows are copies
    # pool(): selection on the rows as given, mean, then the turn at the slot owner's position
    keep_idx, assign = vorta.vorta_bcs_build_index(plan, k, routes)
    pooled = vorta.vorta_bcs_pool(plan, k, routes, keep_idx, assign, rotate=True)
    plain = vorta.vorta_bcs_pool(plan, k, routes, keep_idx, assign, rotate=False)
    torch.cuda.synchronize()
    kh = hnd(k, layout)
    for slot, h in enumerate([1, 3]):
        ki, asg, gap = vo.bcs_select(f64(kh[h])[:L], cfg.grid, cfg.bucket, cfg.keep_num, cfg.keep_den)
        assert gap > 1e-9 and np.array_equal(keep_idx[slot].cpu().numpy(), ki)
        mean = vo.bcs_pool(f64(kh[h])[:L], ki, asg)
        want = np.concatenate([vo.rope_video_rows(mean, spec, ki), f64(kh[h])[L:]])
        assert np.abs(f64(pooled[slot]) - want).max() <= rel * max(1.0, np.abs(want).max())
        assert np.abs(f64(plain[slot])[:len(ki)] - mean).max() <= rel * max(1.0, np.abs(mean).max())


@pytest.mark.parametrize("dtype,d,rope", [("bf16", 128, WAN_ROPE), ("fp32", 64, (16, 24, 24))])
@pytest.mark.parametrize("layout", [1, 0])
def test_small_layers_with_rope_every_route(dtype, d, rope, layout):
    cfg = roped_cfg("rope_small", (5, 6, 9), 4, dtype, (5, 2, 3), [2, 1, 0, 1], d=d, n_text=37, rope=rope)
    check_layer(cfg, cfg.fixed_routes, layout=layout)


def test_rope_with_large_tiles_clipped_grids_and_a_short_period():
    # tiles of 192 tokens (the 8-wavefront window kernel), a grid the tile and the bucket do not
    # divide, theta = 256 (rates that wrap around within the grid), rope spans short of the head
    cfg = roped_cfg("rope_big_tiles", (9, 11, 14), 5, "bf16", (4, 6, 8), [1, 0, 1, 2, 2], n_text=9, rope=HUNYUAN_ROPE[:2] + (40,),
                    theta=256.0)
    check_layer(cfg, cfg.fixed_routes)
    check_layer(cfg, cfg.fixed_routes, layout=0, center_mode=2)


def test_single_layer_config_with_rope():
    base = get_config("single")
    cfg = roped_cfg("single_rope", base.grid, base.heads, "bf16", base.tile, base.fixed_routes, seed=base.seed)
    rows = np.arange(2, cfg.n_tokens, 23)
    plan, out = check_layer(cfg, cfg.fixed_routes, rows=rows)
    # and it is not the layer without the rotation
    q, k, v = make_qkv(cfg, DEV)
    bare = vorta.vorta_routed_attention_layer(vorta.plan_for(base), q, k, v, base.fixed_routes)
    torch.cuda.synchronize()
    assert (out.float() - bare.float()).abs().max().item() > 0.05


@pytest.mark.parametrize("dtype,d,rope", [("bf16", 128, WAN_ROPE), ("fp32", 64, (16, 24, 24))])
def test_soft_mixture_with_rope(dtype, d, rope):
    cfg = roped_cfg("rope_mix", (4, 6, 8), 3, dtype, (2, 3, 4), [0, 1, 2], d=d, n_text=5, rope=rope)
    alpha = np.array([[0.2, 0.5, 0.3], [0.6, 0.1, 0.3], [0.1, 0.1, 0.8]], dtype=np.float32)
    q, k, v = make_qkv(cfg, DEV)
    plan = vorta.plan_for(cfg)
    out = vorta.vorta_soft_mixture_layer(plan, q, k, v, alpha)
    torch.cuda.synchronize()
    want = vo.soft_mixture_layer(f64(q), f64(k), f64(v), alpha.astype(np.float64), spec_of(cfg))
    err = np.abs(f64(out) - want).max()
    say(f"soft mixture with rope {dtype}: max-abs {err:.3e}")
    assert err <= TOL[dtype]


def test_layer_with_rope_equals_its_staged_calls():
    """rope rows -> index -> rotating pool -> attention -> scatter back, call by call, against
    the one-call layer: the same kernels on the same buffers, so equal bit for bit."""
    cfg = roped_cfg("rope_staged", (6, 8, 8), 5, "bf16", (2, 4, 4), [0, 1, 2, 2, 1], n_text=10)
    routes = np.array(cfg.fixed_routes, dtype=np.uint8)
    q, k, v = make_qkv(cfg, DEV)
    plan = vorta.plan_for(cfg)
    out = vorta.vorta_routed_attention_layer(plan, q, k, v, routes)
    q_r, k_r = vorta.vorta_rope_apply(plan, q, routes), vorta.vorta_rope_apply(plan, k, routes)
    keep_idx, assign, q_c, k_c, v_c = vorta.vorta_bcs_select_pool(plan, q, k, v, routes)
    o_c, staged = torch.empty_like(q_c), torch.zeros_like(q)
    vorta.vorta_attention_routed(plan, routes, q=q_r, k=k_r, v=v, out=staged, q_c=q_c, k_c=k_c, v_c=v_c, o_c=o_c)
    vorta.vorta_scatter_back(plan, routes, None, o_c, assign, staged)
    torch.cuda.synchronize()
    assert torch.equal(out, staged)


def test_wan480p_sized_layer_with_rope_hard_routed_and_mixed():
    """The 480p grid (32,760 tokens, 72-token tiles, grouped window items, fused selection +
    pooling) with a Wan-style rotary split: three heads, one per route, then the same three heads
    under Eq. 5 -- sampled rows of every head against the oracle."""
    base = get_config("wan480p")
    cfg = LayerConfig("wan480p_rope", base.grid, 3, 128, "bf16", base.tile, base.window, seed=83,
                      fixed_routes=(0, 1, 2), rope_dims=WAN_ROPE)
    L = cfg.n_video
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.choice(L, 384, replace=False), np.arange(0, 72), np.arange(L - 3, L)]))
    say("wan480p-sized layer with rope: hard routing")
    plan, out = check_layer(cfg, cfg.fixed_routes, rows=rows)
    q, k, v = make_qkv(cfg, DEV)
    alpha = np.array([[0.5, 0.3, 0.2], [0.1, 0.6, 0.3], [0.3, 0.3, 0.4]], dtype=np.float32)
    say("wan480p-sized layer with rope: soft mixture")
    mixed = vorta.vorta_soft_mixture_layer(plan, q, k, v, alpha)
    torch.cuda.synchronize()
    want = vo.soft_mixture_layer(f64(q), f64(k), f64(v), alpha.astype(np.float64), spec_of(cfg), rows)
    err = np.abs(f64(mixed[:, torch.as_tensor(rows, device=DEV)]) - want).max(axis=(1, 2))
    say(f"  soft mixture max-abs per head {np.array2string(err, precision=4)}")
    assert err.max() <= TOL["bf16"]
