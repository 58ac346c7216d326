"""The layer entry point that allocates nothing (vorta_routed_attention_layer_static) against
vorta_routed_attention_layer: same kernels over the library's static scratch instead of a caller
workspace, so the outputs must agree bit for bit -- on two calls in a row, the second on a
smaller layer, whose buffers then lie inside what the first call left in the scratch."""
import sys

import numpy as np
import pytest
import torch

import paper_2505_18809_amd as vorta
from synth_inputs import LayerConfig, get_config, make_qkv, make_routes

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_both(cfg, routes, layout=1):
    q, k, v = make_qkv(cfg, DEV, layout)
    plan = vorta.plan_for(cfg, layout=layout)
    want = vorta.vorta_routed_attention_layer(plan, q, k, v, routes)       # allocates its workspace, uploads the tables
    torch.cuda.synchronize()
    vorta.vorta_plan_upload(plan)                                          # idempotent set-up call
    got = torch.full_like(q, float("nan"))
    before = torch.cuda.memory_allocated()
    vorta.vorta_routed_attention_layer_static(plan, q, k, v, routes, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return plan, want, got


def test_static_scratch_layer_matches_the_workspace_layer_twice_in_a_row():
    big = get_config("single")                                             # 3,072 tokens, 8 heads: 4.8 MB of scratch
    routes_big = make_routes(big).numpy()
    say("static scratch: single-layer config")
    plan, want, got = run_both(big, routes_big)
    assert vorta.vorta_workspace_bytes(plan, routes_big) <= vorta.VORTA_STATIC_SCRATCH_BYTES
    assert torch.equal(got, want)
    small = LayerConfig("small_after_big", (5, 7, 9), 5, 128, "bf16", (2, 3, 4), (3, 3, 3), seed=19, n_text=11,
                        fixed_routes=(2, 1, 0, 2, 1))
    say("static scratch: smaller layer right after it")
    _, want, got = run_both(small, np.array(small.fixed_routes, dtype=np.uint8), layout=0)
    assert torch.equal(got, want)
    tiny = get_config("tiny")                                              # fp32: tile-ordered copies live in the scratch too
    say("static scratch: fp32 layer")
    _, want, got = run_both(tiny, np.array([1, 2], dtype=np.uint8))
    assert torch.equal(got, want)


def test_static_scratch_layer_refuses_what_it_cannot_do():
    cfg = get_config("single")
    routes = make_routes(cfg).numpy()
    q, k, v = make_qkv(cfg, DEV)
    out = torch.empty_like(q)
    fresh = vorta.plan_for(cfg)
    with pytest.raises(vorta.VortaError) as e:                             # tables not uploaded: it never uploads itself
        vorta.vorta_routed_attention_layer_static(fresh, q, k, v, routes, out)
    assert e.value.code == -1 and "vorta_plan_upload" in str(e.value)
    large = get_config("wan480p")                                          # needs 268 MB of scratch
    plan = vorta.plan_for(large)
    vorta.vorta_plan_upload(plan)
    shape = plan.user_shape()
    x = torch.empty(shape, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(vorta.VortaError) as e:
        vorta.vorta_routed_attention_layer_static(plan, x, x, x, make_routes(large).numpy(), torch.empty_like(x))
    assert e.value.code == -4
