#!/usr/bin/env python3
"""Benchmark of the routed attention layer on one MI355X.

A step is one pass of the whole hot path -- core-set selection and pooling, the routed
attention launches (window rows gathered through the tile permutation), unpool / scatter back
-- over one seeded synthetic layer, with Q/K/V already resident in HBM.  Prints ONE JSON line.

  value       effective TFLOP/s of the whole layer call: FLOPs of the two contractions
              actually required by each head's route (padding and softmax not counted)
              / wall time per step
  roofline    the fused attention kernel alone, timed with events on its stream in a second
              pass over the same buffers, against the dense bf16 MFMA peak
  cpu_baseline the fp64 NumPy oracle on a bounded sample of the same layer's rows,
              extrapolated to one layer (context, not a target)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "ms per routed attention layer + effective TFLOP/s (% MFMA peak) at 75.6k tokens"
MFMA_PEAK_TFLOPS = {"bf16": 2516.6, "fp32": 157.3}      # MI355X dense peaks
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "layer_wan720p_hbm_traffic.txt")


def profiled_traffic(kernel, workload, layout):
    """HBM-side bytes per launch of `kernel`, read from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE runs of this same command, scaled by what the counters read for a
    plain 1 GiB copy).  It is a recorded figure, not a live one: it is reported only for the
    command the profile was taken with (wan720p, HND layout) and names its source; None if the
    summary is missing or has no row for the kernel."""
    if workload != "wan720p" or layout != 1 or not os.path.exists(TRAFFIC_PROFILE):
        return None
    for line in open(TRAFFIC_PROFILE):
        if line.startswith(kernel):
            nums = [int(tok.replace(",", "")) for tok in line[len(kernel):].replace("/", " ").split()
                    if tok.replace(",", "").isdigit()]
            if len(nums) >= 5:            # FETCH raw, FETCH KiB, WRITE KiB, algorithmic read KiB, algorithmic write KiB
                return {"bytes": (nums[1] + nums[2]) * 1024, "algorithmic_bytes": (nums[3] + nums[4]) * 1024,
                        "source": os.path.relpath(TRAFFIC_PROFILE, ROOT)}
    return None


def layer_flops(cfg, plan, routes):
    """QK^T and PV multiply-adds (2 FLOP each) each route has to do; returns per-route totals."""
    import numpy as np
    import paper_2505_18809_amd as vorta
    d, N, Lt = cfg.head_dim, cfg.n_tokens, cfg.n_text
    # window heads: every query of a tile sees the keys of the tile's run list (text keys included);
    # counted from the plan's host tables, so clipped edge tiles and truncated windows are exact
    runs, n_runs = vorta.vorta_window_runs(plan)
    keys = np.array([runs[t, :n_runs[t], 1].sum() for t in range(plan.n_tiles)], dtype=np.float64)
    rows = np.diff(vorta.vorta_tile_row0(plan)).astype(np.float64)
    per_head = [4.0 * N * N * d,
                4.0 * d * (float((rows * keys).sum()) + Lt * N),
                4.0 * (plan.n_core + Lt) ** 2 * d]
    counts = [int((routes == r).sum()) for r in range(3)]
    return [per_head[r] * counts[r] for r in range(3)], per_head, counts


def cpu_baseline(cfg, q, k, v, routes, total_flops, per_head_flops, counts, budget_s=20.0):
    """Time the oracle on a few rows of one head per route and scale to the layer."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import vorta_oracle as vo

    spec = vo.LayerSpec(grid=cfg.grid, tile=cfg.tile, window=cfg.window, bucket=cfg.bucket,
                        keep_num=cfg.keep_num, keep_den=cfg.keep_den, n_text=cfg.n_text)
    N, L = cfg.n_tokens, cfg.n_video
    rng = np.random.default_rng(0)
    layer_s, sample = 0.0, []
    n_rows = {0: 2048, 1: 4096, 2: 4096}      # about 10-20 s of CPU work on the GPU machine's host share
    for r in range(3):
        if counts[r] == 0:
            continue
        h = int(np.nonzero(routes == r)[0][0])
        Q, K, V = (t[h].double().cpu().numpy() for t in (q, k, v))
        rows = np.sort(rng.choice(N, min(n_rows[r], N), replace=False))
        fixed = 0.0
        t0 = time.perf_counter()
        if r == 2:
            index = vo.bcs_select(K[:L], cfg.grid, cfg.bucket, cfg.keep_num, cfg.keep_den)
            fixed = time.perf_counter() - t0            # whole-head cost, not per row
            t0 = time.perf_counter()
            vo.coreset_attention(Q, K, V, spec, rows, index=index)
        else:
            vo.head_attention(r, Q, K, V, spec, rows)
        per_row = (time.perf_counter() - t0) / len(rows)
        # a core-set row stands for the tokens merged into it: L_c + Lt distinct rows per head
        head_rows = (L // 2 + cfg.n_text) if r == 2 and cfg.keep_den == 2 * cfg.keep_num else N
        layer_s += counts[r] * (fixed + per_row * head_rows)
        sample.append(f"route {r}: {len(rows)} rows of head {h}")
    threads = max([i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"] or [1])
    return {"value": total_flops / layer_s / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "ms_per_layer_extrapolated": layer_s * 1e3,
            "sample": "fp64 NumPy oracle, " + "; ".join(sample) + "; per-row time scaled to all rows and heads"}


def mfma_probe(torch, dev):
    """Matrix-pipe rate with nothing else running, per operand distribution (context for the
    roofline fraction: the nominal peak assumes the nominal clock, the sustained clock depends
    on how many operand bits toggle)."""
    from paper_2505_18809_amd import probe
    out = {}
    gen = torch.Generator(device="cpu").manual_seed(1)
    kinds = {
        "zeros": torch.zeros(16 * 64 * 8),
        "constant_1.0": torch.ones(16 * 64 * 8),
        "normal": torch.randn(16 * 64 * 8, generator=gen),
    }
    def rate(ops, shape=32, vector_ops=0):
        iters, wgs = 4000, 256 * 4
        probe.mfma_probe_rate(ops, 200, wgs, shape, vector_ops)            # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops, _, clocks = probe.mfma_probe_rate(ops, iters, wgs, shape, vector_ops)
        e1.record()
        torch.cuda.synchronize()
        c = clocks.cpu().tolist()
        return {"TFLOP/s": flops / (e0.elapsed_time(e1) * 1e-3) / 1e12,
                "shader_clock_MHz": c[0] / max(c[1], 1) * 100.0}

    for name, vals in kinds.items():
        out[name] = rate(vals.to(torch.bfloat16).to(dev))
    # the other bf16 shape on the same random operands (what the power limit leaves of it), and, on
    # zero operands (no power limit), what 2, 3 and 4 vector instructions per 16 cycles of
    # matrix-pipe time leave of either shape's rate: the vector issue port's share of a matrix instruction
    out["normal_16x16x32"] = rate(kinds["normal"].to(torch.bfloat16).to(dev), shape=16)
    zeros = kinds["zeros"].to(torch.bfloat16).to(dev)
    out["zeros_with_vector_ops_TFLOPs"] = {
        f"{name}": {str(kv): round(rate(zeros, shape, kv)["TFLOP/s"], 1) for kv in (0, 2, 3, 4)}
        for name, shape in (("32x32x16", 32), ("16x16x32", 16))}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="wan720p")
    ap.add_argument("--layout", type=int, default=1, help="1 = [heads][N][d], 0 = [N][heads][d]")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--zero-operands", action="store_true",
                    help="also time the dominant kernel's launch on all-zero Q/K/V (what the power limit costs on real data)")
    ap.add_argument("--routes-alone", action="store_true",
                    help="also time the heads of each route alone (per-route TFLOP/s); off by default like --zero-operands")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size reference for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)")

    import numpy as np
    import torch
    import paper_2505_18809_amd as vorta
    from synth_inputs import get_config, make_qkv, make_routes

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the library has no CPU path")
    dev = "cuda:0"
    cfg = get_config(args.workload)
    routes = make_routes(cfg).numpy()
    q, k, v = make_qkv(cfg, dev, args.layout)
    plan = vorta.plan_for(cfg, layout=args.layout)
    out = torch.empty_like(q)
    ws = torch.empty(vorta.vorta_workspace_bytes(plan, routes), dtype=torch.uint8, device=dev)
    per_route, per_head, counts = layer_flops(cfg, plan, routes)
    flops = sum(per_route)

    def step():
        vorta.vorta_routed_attention_layer(plan, q, k, v, routes, out=out, workspace=ws)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)            # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # second pass: the same launches issued stage by stage, events around each stage
    off = vorta.vorta_workspace_layout(plan, routes)
    n_win, n_lr = counts[1], counts[2]
    row = cfg.head_dim * plan.elem_bytes
    def buf(i, heads, rows):
        return ws[off[i]: off[i] + heads * rows * row].view(q.dtype).view(heads, rows, cfg.head_dim)
    q_t, k_t, v_t, o_t = (buf(i, n_win, plan.n_tokens) for i in range(4))
    q_c, k_c, v_c, o_c = (buf(i, n_lr, plan.n_core_tokens) for i in range(4, 8))
    keep_idx = ws[off[8]: off[8] + n_lr * plan.n_core * 4].view(torch.int32).view(n_lr, plan.n_core)
    assign = ws[off[9]: off[9] + n_lr * plan.n_video * 4].view(torch.int32).view(n_lr, plan.n_video)
    # what the layer call issues: with bf16 the window kernel gathers rows through the tile
    # permutation, so there is no reorder pass and no tile-ordered copy
    gather = cfg.dtype == "bf16"
    tiled = {} if gather else dict(q_t=q_t, k_t=k_t, v_t=v_t, o_t=o_t)
    stages = {}
    if not gather:
        stages["reorder_to_tiles"] = lambda: [vorta.vorta_reorder_to_tiles(plan, s, routes, d) for s, d in ((q, q_t), (k, k_t), (v, v_t))]
    stages.update({
        "bcs_select_pool": lambda: vorta.vorta_bcs_select_pool(plan, q, k, v, routes, keep_idx, assign, q_c, k_c, v_c),
        "attention_routed": lambda: vorta.vorta_attention_routed(plan, routes, q=q, k=k, v=v, out=out, q_c=q_c, k_c=k_c,
                                                                  v_c=v_c, o_c=o_c, **tiled),
        "scatter_back": lambda: vorta.vorta_scatter_back(plan, routes, None if gather else o_t, o_c, assign, out),
    })
    stage_ms = {name: 0.0 for name in stages}
    events = []
    for _ in range(args.steps):
        for name, fn in stages.items():
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            events.append((name, e0, e1))
    torch.cuda.synchronize()
    for name, e0, e1 in events:
        stage_ms[name] += e0.elapsed_time(e1) / args.steps

    # algorithmic bytes of the memory passes (read + write of the rows each pass must move)
    N, L, Lc = plan.n_tokens, plan.n_video, plan.n_core
    pass_bytes = {
        "reorder_to_tiles": 2 * 3 * n_win * N * row,
        # Q, K, V read once, three pooled tensors and the two index arrays written
        "bcs_select_pool": 3 * n_lr * (N + plan.n_core_tokens) * row + n_lr * (Lc + L) * 4,
        "scatter_back": (0 if gather else 2 * n_win * N * row) + n_lr * (N + plan.n_core_tokens) * row + n_lr * L * 4,
    }
    attn_ms = stage_ms["attention_routed"]
    peak = MFMA_PEAK_TFLOPS[cfg.dtype]

    # Attention of a subset of the heads alone: a plan that holds only those heads reproduces their
    # items of the layer's launches exactly; timed with events on the stream of the launches.
    def heads_alone(mask, zero=False):
        sel = np.nonzero(mask)[0]
        sub_routes = np.ascontiguousarray(routes[sel])
        sub_plan = vorta.plan_for(cfg, layout=args.layout, heads=len(sel))
        idx = torch.as_tensor(sel, device=dev)
        hd = 0 if args.layout == 1 else 1
        sq, sk, sv = (t.index_select(hd, idx).contiguous() for t in (q, k, v))
        so = torch.empty_like(sq)
        kw = dict(q=sq, k=sk, v=sv, out=so)
        n_core = int((sub_routes == 2).sum())
        pooled = ()
        if n_core:
            sws = torch.empty(vorta.vorta_workspace_bytes(sub_plan, sub_routes), dtype=torch.uint8, device=dev)
            vorta.vorta_routed_attention_layer(sub_plan, sq, sk, sv, sub_routes, out=so, workspace=sws)   # fills the pooled buffers
            soff = vorta.vorta_workspace_layout(sub_plan, sub_routes)
            def sbuf(i):
                return sws[soff[i]: soff[i] + n_core * plan.n_core_tokens * row].view(q.dtype).view(n_core, plan.n_core_tokens, cfg.head_dim)
            pooled = (sbuf(4), sbuf(5), sbuf(6))
            kw.update(q_c=pooled[0], k_c=pooled[1], v_c=pooled[2], o_c=sbuf(7))

        def timed(n):
            vorta.vorta_attention_routed(sub_plan, sub_routes, **kw)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                vorta.vorta_attention_routed(sub_plan, sub_routes, **kw)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        res = {"ms": timed(args.steps)}
        # The same launch on all-zero operands: the same instructions and cycle count, but no
        # operand bit toggles, so the power limit does not hold the clock down.  A diagnostic
        # of what the limit costs on real data, not a throughput claim.
        if zero:
            for t in (sq, sk, sv) + pooled:
                t.zero_()
            res["zero_ms"] = timed(3)
        return res

    # dominant kernel alone: the dense and core-set heads of this layer form one launch of the
    # pipelined kernel (the window heads are the launches after it)
    dom = {"kernel": "attn_f32_kernel", "ms": attn_ms, "flops": flops}
    win_ms = None
    route_alone = {}
    if cfg.dtype == "bf16":
        if counts[0] + counts[2] > 0:
            # (zero operands: off by default, so that a profile of the default command holds launches of one kind)
            dom = {"kernel": "attn_bf16_pipe_kernel<false, 8>", "flops": per_route[0] + per_route[2],
                   **heads_alone(routes != 1, zero=args.zero_operands)}
        # the window heads alone (their tiles are the attention call's later launches; their text
        # rows, if the layer has text tokens, ride in a short launch of the pipelined kernel)
        if counts[1] > 0:
            win_ms = heads_alone(routes == 1)["ms"]
        # and, on request, every route alone (launches of the dominant kernel on other head sets:
        # off by default for the same reason as the zero operands)
        for r, name in enumerate(("full", "window", "core-set")):
            if args.routes_alone and counts[r] > 0:
                r_ms = win_ms if r == 1 else heads_alone(routes == r)["ms"]
                route_alone[name] = {"heads": counts[r], "ms": r_ms, "TFLOP/s": per_route[r] / (r_ms * 1e-3) / 1e12}
    achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
    traffic = profiled_traffic(dom["kernel"], args.workload, args.layout)
    result = {
        "metric": METRIC,
        "value": flops / (ms * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms,
        "ms_per_layer": ms,
        "mfma_peak_frac": flops / (ms * 1e-3) / 1e12 / peak,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: grid {cfg.grid} = {cfg.n_video} video + {cfg.n_text} text tokens, "
                               f"{cfg.heads} heads x {cfg.head_dim}, tiles {cfg.tile}, window {cfg.window} tiles, "
                               f"bucket {cfg.bucket} r={cfg.keep_num}/{cfg.keep_den}",
                   "routes_full_window_coreset": counts, "layout": "HND" if args.layout == 1 else "NHD",
                   "flops_per_layer": flops},
        "roofline": {"bound": "mfma", "kernel": dom["kernel"],
                     "launch": f"{counts[0]} dense + {counts[2]} core-set heads of the layer (the window heads are a separate launch)",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "flops_per_launch": dom["flops"], "ms_per_launch": dom["ms"],
                     "traffic": traffic["bytes"] if traffic else None,
                     "traffic_algorithmic": traffic["algorithmic_bytes"] if traffic else None,
                     "traffic_source": traffic["source"] if traffic else None},
        "dominant_kernel_on_zero_operands": ({"ms_per_launch": dom["zero_ms"],
                                              "TFLOP/s": dom["flops"] / (dom["zero_ms"] * 1e-3) / 1e12,
                                              "frac": dom["flops"] / (dom["zero_ms"] * 1e-3) / 1e12 / peak,
                                              "note": "same launch, all-zero Q/K/V: same cycle count, clock not held down by the power limit"}
                                             if "zero_ms" in dom else None),
        "stages_ms": stage_ms,
        # the attention call is two launches, each timed alone on a plan holding only its heads
        "attention_launches": {
            "dense+core-set": {"ms": dom["ms"], "TFLOP/s": dom["flops"] / (dom["ms"] * 1e-3) / 1e12},
            "window": ({"ms": win_ms, "TFLOP/s": per_route[1] / (win_ms * 1e-3) / 1e12} if win_ms else None),
        },
        "routes_alone": route_alone or None,
        "memory_passes_GBps": {n: pass_bytes[n] / (stage_ms[n] * 1e-3) / 1e9 for n in pass_bytes if stage_ms.get(n, 0) > 0},
    }
    if cfg.dtype == "bf16":
        result["mfma_probe"] = mfma_probe(torch, dev)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, q if args.layout == 1 else q.transpose(0, 1),
                                              k if args.layout == 1 else k.transpose(0, 1),
                                              v if args.layout == 1 else v.transpose(0, 1),
                                              routes, flops, per_head, counts)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
