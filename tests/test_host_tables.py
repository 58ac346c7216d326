"""Host-side logic of libvorta against the oracle (bit-exact integers) and the ABI surface.
No compute call is made: these run without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2505_18809_amd as vorta
from oracle import vorta_oracle as vo
from synth_inputs import CONFIGS, get_config, make_routes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "vorta.h")).read()
    declared = set(re.findall(r"\b(vorta_[a-z0-9_]+)\s*\(", header))
    assert declared == set(vorta.SYMBOLS)
    lib = vorta.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.vorta_strerror(-2) == b"unsupported shape"


def test_probe_library_loads_and_rejects_bad_arguments():
    """The benchmark's matrix-rate probe is a library of its own; without a GPU only its
    argument checks can run (they return before any launch)."""
    from paper_2505_18809_amd import probe
    lib = ctypes.CDLL(probe.PROBE_LIB_PATH)
    fn = lib.mfma_probe_rate
    fn.restype = ctypes.c_int
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(256)
    assert fn(null, 1, 1, 32, 0, one, one, null) == -1          # no operands
    assert fn(one, 0, 1, 32, 0, one, one, null) == -1           # no trips
    assert fn(one, 1, 1, 8, 0, one, one, null) == -1            # unknown shape
    assert fn(one, 1, 1, 16, 1, one, one, null) == -1           # unknown number of vector instructions
    assert not hasattr(vorta.load_library(), "mfma_probe_rate")  # and it is not part of libvorta


def test_struct_sizes_match_the_header():
    # 8 scalars + 3+3 ints + center_mode + 3 ints + 2 ints + float + 3 ints + float = 25 four-byte fields
    assert ctypes.sizeof(vorta.binding.vorta_layer_desc) == 25 * 4
    assert ctypes.sizeof(vorta.binding.vorta_attn_io) == 12 * 8


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_plan_geometry(cfg):
    plan = vorta.plan_for(cfg)
    assert plan.n_video == cfg.n_video and plan.n_tokens == cfg.n_tokens
    assert plan.tiles == vo.tile_grid(cfg.grid, cfg.tile)
    assert plan.tile_tokens == int(np.prod(cfg.tile))
    assert 2 * plan.n_core == cfg.n_video                 # ratio 0.5 halves every benchmark grid
    assert plan.n_core_tokens == plan.n_core + cfg.n_text
    assert plan.window_key_tiles == int(np.prod([min(3, n) for n in plan.tiles]))


@pytest.mark.parametrize("grid,tile", [((4, 8, 8), (2, 4, 4)), ((3, 4, 6), (1, 2, 3)), ((12, 16, 16), (4, 4, 4)),
                                       ((5, 7, 6), (2, 3, 4)), ((3, 5, 5), (4, 2, 6)), ((20, 9, 10), (6, 9, 8))])
def test_tile_permutation_matches_get_tile_id_3d(grid, tile):
    """Also on grids the tile does not divide (clipped edge tiles)."""
    plan = vorta.vorta_plan_create(grid, 1, 128, "bf16", tile, (3, 3, 3))
    perm = vorta.vorta_tile_permutation(plan)
    row0 = vorta.vorta_tile_row0(plan)
    L = int(np.prod(grid))
    assert sorted(perm) == list(range(L))
    n = vo.tile_grid(grid, tile)
    assert plan.tiles == n and len(row0) == plan.n_tiles + 1 and row0[0] == 0 and row0[-1] == L
    tile_of_row = np.searchsorted(row0, np.arange(L), side="right") - 1
    for i in range(L):
        tid = vo.get_tile_id_3d(i, grid, tile)
        assert tile_of_row[perm[i]] == np.ravel_multi_index(tid, n)
    # inside a tile, positions follow raster order of the tokens
    for t in range(plan.n_tiles):
        members = np.nonzero(tile_of_row[perm] == t)[0]
        assert (np.diff(perm[members]) == 1).all() and perm[members[0]] == row0[t]
    if all(g % t == 0 for g, t in zip(grid, tile)):
        assert (row0 == np.arange(plan.n_tiles + 1) * int(np.prod(tile))).all()


MODES = {"clamp": 0, "identity": 1, "block": 2}


@pytest.mark.parametrize("mode", ["clamp", "identity", "block"])
@pytest.mark.parametrize("window", [(1, 1, 1), (3, 3, 3), (1, 3, 5), (5, 2, 3)])
@pytest.mark.parametrize("grid,tile", [((4, 6, 6), (2, 2, 3)), ((5, 7, 6), (2, 3, 4))], ids=["divisible", "clipped"])
def test_window_boxes_and_runs_expand_to_algorithm_1_mask(window, mode, grid, tile):
    n_text = 5
    plan = vorta.vorta_plan_create(grid, 1, 128, "bf16", tile, window, n_text=n_text,
                                   center_mode=MODES[mode])
    M = vo.sta_mask_dense(grid, tile, window, mode)
    perm = vorta.vorta_tile_permutation(plan)
    inv = np.argsort(perm)
    boxes = vorta.vorta_window_boxes(plan)
    runs, n_runs = vorta.vorta_window_runs(plan)
    n = plan.tiles
    L = plan.n_video
    for i in range(L):
        qt = np.ravel_multi_index(vo.get_tile_id_3d(i, grid, tile), n)
        lo, hi = boxes[qt, 0::2], boxes[qt, 1::2]
        from_box = np.array([all(lo[a] <= vo.get_tile_id_3d(j, grid, tile)[a] <= hi[a] for a in range(3))
                             for j in range(L)])
        assert (from_box == M[i]).all()
        rows = np.concatenate([np.arange(s, s + c) for s, c in runs[qt, :n_runs[qt]]])
        assert len(set(rows)) == len(rows)
        video = np.sort(inv[rows[rows < L]])
        assert (video == np.nonzero(M[i])[0]).all()
        assert sorted(rows[rows >= L]) == list(range(L, L + n_text))       # text keys always visible
        assert (runs[qt, :n_runs[qt], 1] > 0).all()


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_geometries_expand_to_algorithm_1_mask(seed):
    """Random small grids, tiles (dividing the grid or not), windows and centre rules: the run
    table of every query tile, mapped back through the tile permutation, is exactly the row of
    Algorithm 1's mask; runs are disjoint, non-empty and ascending."""
    rng = np.random.default_rng(4000 + seed)
    grid = tuple(int(x) for x in rng.integers(1, 8, 3))
    tile = tuple(int(x) for x in rng.integers(1, 5, 3))
    window = tuple(int(x) for x in rng.choice([1, 2, 3, 5, 7], 3))
    mode = ["clamp", "identity", "block"][seed % 3]
    n_text = int(rng.choice([0, 3]))
    plan = vorta.vorta_plan_create(grid, 1, 128, "bf16", tile, window, n_text=n_text, center_mode=seed % 3)
    L = plan.n_video
    inv = np.argsort(vorta.vorta_tile_permutation(plan))
    row0 = vorta.vorta_tile_row0(plan)
    runs, n_runs = vorta.vorta_window_runs(plan)
    n = vo.tile_grid(grid, tile)
    assert plan.tiles == n
    for i in range(L):
        qt = int(np.ravel_multi_index(vo.get_tile_id_3d(i, grid, tile), n))
        r = runs[qt, :n_runs[qt]]
        assert (r[:, 1] > 0).all() and (r[1:, 0] > r[:-1, 0] + r[:-1, 1] - 1).all()     # ascending, disjoint
        rows = np.concatenate([np.arange(s0, s0 + c) for s0, c in r])
        want = np.nonzero(vo.sta_mask_row(i, grid, tile, window, mode))[0]
        assert (np.sort(inv[rows[rows < L]]) == want).all(), (grid, tile, window, mode, i)
        assert sorted(rows[rows >= L]) == list(range(L, L + n_text))
        assert row0[qt] <= np.nonzero(inv == i)[0][0] < row0[qt + 1]


def test_block_centres_follow_the_hand_worked_fixture():
    """The library's run table under VORTA_CENTER_BLOCK against the hand-worked mask in
    tests/golden (7 tiles, window 3: blocks {0,1,2} {3,4,5} {6})."""
    from test_oracle_pins import read_mask_fixture
    want = read_mask_fixture("sta_mask_1x1x14_tile2_win3_block.txt")["block"]
    plan = vorta.vorta_plan_create((1, 1, 14), 1, 128, "bf16", (1, 1, 2), (1, 1, 3), center_mode=2)
    boxes = vorta.vorta_window_boxes(plan)
    assert [tuple(b[4:]) for b in boxes] == [(0, 2)] * 3 + [(3, 5)] * 3 + [(6, 6)]
    runs, n_runs = vorta.vorta_window_runs(plan)
    for i in range(14):                                   # one tile row: tile order = raster order
        got = np.zeros(14, dtype=bool)
        for s0, c in runs[i // 2, :n_runs[i // 2]]:
            got[s0:s0 + c] = True
        assert (got == want[i]).all()


@pytest.mark.parametrize("tile,bucket", [((2048, 2048, 2048), (2, 3, 2)), ((70000, 70000, 1), (1000, 1, 1)),
                                         ((2 ** 31 - 1, 3, 2 ** 31 - 1), (2 ** 31 - 1, 2 ** 31 - 1, 2 ** 31 - 1)),
                                         ((5, 8, 3), (4, 1, 1))])
def test_tiles_and_buckets_larger_than_the_grid_are_clipped_to_it(tile, bucket):
    """A tile (bucket) extent beyond its axis means one tile (bucket) along that axis: the plan
    must equal the plan made with the extents clipped by hand -- no overflowing products, no
    zero-sized tiles."""
    grid = (4, 8, 8)
    clip = lambda t: tuple(min(x, g) for x, g in zip(t, grid))
    if int(np.prod(clip(bucket))) > 64:
        with pytest.raises(vorta.VortaError) as e:
            vorta.vorta_plan_create(grid, 2, 128, "bf16", tile, (3, 3, 3), bucket=bucket)
        assert e.value.code == -2
        bucket = (2, 3, 2)
    a = vorta.vorta_plan_create(grid, 2, 128, "bf16", tile, (3, 3, 2 ** 31 - 1), bucket=bucket, n_text=3)
    b = vorta.vorta_plan_create(grid, 2, 128, "bf16", clip(tile), (3, 3, 99), bucket=clip(bucket), n_text=3)
    assert a.tile_tokens == int(np.prod(clip(tile))) and a.tile_tokens <= a.n_video
    for name in ("tiles", "n_tiles", "tile_tokens", "window_key_tiles", "max_runs", "n_buckets", "n_core"):
        assert getattr(a, name) == getattr(b, name), name
    assert (vorta.vorta_tile_permutation(a) == vorta.vorta_tile_permutation(b)).all()
    assert (vorta.vorta_tile_row0(a) == vorta.vorta_tile_row0(b)).all()
    ra, rb = vorta.vorta_window_runs(a), vorta.vorta_window_runs(b)
    assert (ra[0] == rb[0]).all() and (ra[1] == rb[1]).all()
    assert (vorta.vorta_bcs_slot_bases(a) == vorta.vorta_bcs_slot_bases(b)).all()
    perm = vorta.vorta_tile_permutation(a)
    n = vo.tile_grid(grid, clip(tile))
    row0 = vorta.vorta_tile_row0(a)
    for i in range(0, a.n_video, 7):
        t = int(np.ravel_multi_index(vo.get_tile_id_3d(i, grid, tile), n))
        assert row0[t] <= perm[i] < row0[t + 1]


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("grid,tile,window", [((21, 45, 80), (3, 5, 8), (3, 3, 3)), ((21, 30, 52), (3, 6, 4), (3, 3, 3)),
                                              ((5, 7, 6), (2, 3, 4), (3, 1, 5)), ((4, 8, 8), (1, 1, 1), (3, 3, 3)),
                                              ((12, 16, 16), (4, 4, 4), (3, 3, 3)), ((9, 11, 14), (4, 6, 8), (3, 3, 3))])
def test_window_items_group_tiles_with_identical_key_sets(grid, tile, window, mode):
    """Every tile in exactly one item; the tiles of an item have the same run list (so one key
    stream serves them), at most three tiles and 256 rows; items of more than 128 rows come first."""
    plan = vorta.vorta_plan_create(grid, 1, 128, "bf16", tile, window, n_text=3, center_mode=mode)
    big, small = vorta.vorta_window_items(plan)
    if plan.tile_tokens > 128:
        assert len(big) == 0 and len(small) == 0
        return
    runs, n_runs = vorta.vorta_window_runs(plan)
    rows_of = np.diff(vorta.vorta_tile_row0(plan))
    seen = []
    for items, is_big in ((big, True), (small, False)):
        assert (np.diff(items[:, 0]) > 0).all()
        for it in items:
            tiles = list(it[:it[3]])
            assert 1 <= it[3] <= 3 and tiles == sorted(tiles)
            rows = int(rows_of[tiles].sum())
            assert rows <= 256 and (rows > 128) == is_big
            for t in tiles[1:]:
                assert n_runs[t] == n_runs[tiles[0]] and (runs[t, :n_runs[t]] == runs[tiles[0], :n_runs[t]]).all()
            seen += tiles
    assert sorted(seen) == list(range(plan.n_tiles))
    if mode == 0 and grid == (21, 45, 80):
        # clamped 3x3x3 window on 7x9x10 tiles: only the 3x5x6 interior tiles have a key set of their own
        assert len(small) == 90 and len(big) == 270
    if mode == 1 and window == (3, 3, 3) and min(plan.tiles) >= 3:
        assert len(big) == 0 and len(small) == plan.n_tiles      # identity centres: all key sets differ


def test_window_covering_the_grid_is_one_run():
    cfg = get_config("tiny")
    plan = vorta.plan_for(cfg)
    runs, n_runs = vorta.vorta_window_runs(plan)
    assert (n_runs == 1).all() and (runs[:, 0] == [0, 256]).all()
    big = vorta.plan_for(get_config("wan720p"))
    runs, n_runs = vorta.vorta_window_runs(big)
    assert big.max_runs == 9 and (n_runs == 9).all()
    assert (runs[:, :, 1] == 3 * 120).all()


@pytest.mark.parametrize("grid,bucket,num,den", [((4, 8, 8), (2, 3, 2), 1, 2), ((5, 7, 3), (2, 3, 2), 1, 2),
                                                  ((4, 6, 6), (2, 2, 2), 1, 4), ((3, 3, 3), (3, 3, 3), 3, 4),
                                                  ((2, 3, 4), (1, 1, 1), 1, 2), ((4, 4, 4), (2, 2, 1), 1, 1)])
def test_bcs_slot_bases_match_oracle_bucket_walk(grid, bucket, num, den):
    plan = vorta.vorta_plan_create(grid, 1, 128, "bf16", (1, 1, 1), (1, 1, 1), bucket=bucket, keep_num=num,
                                   keep_den=den)
    sb = vorta.vorta_bcs_slot_bases(plan)
    want = [0]
    for idx, _ in vo.bcs_buckets(grid, bucket):
        want.append(want[-1] + len(idx) - vo.bcs_prune_count(len(idx), num, den))
    assert list(sb) == want and plan.n_core == want[-1] and plan.n_buckets == len(want) - 1


def test_route_partition_and_select():
    cfg = get_config("wan720p")
    plan = vorta.plan_for(cfg)
    routes = make_routes(cfg).numpy()
    heads, counts = vorta.vorta_route_partition(plan, routes)
    assert list(counts) == [6, 18, 16]
    want = [h for r in range(3) for h in range(cfg.heads) if routes[h] == r]
    assert list(heads) == want
    with pytest.raises(vorta.VortaError) as e:
        vorta.vorta_route_partition(plan, np.full(cfg.heads, 3, dtype=np.uint8))
    assert e.value.code == -5
    for wrong in (routes[:2], np.concatenate([routes, routes])):      # a route vector of the wrong length
        with pytest.raises(vorta.VortaError) as e:
            vorta.vorta_route_partition(plan, wrong)
        assert e.value.code == -1
        with pytest.raises(vorta.VortaError) as e:
            vorta.vorta_workspace_bytes(plan, wrong)
        assert e.value.code == -1
    rng = np.random.default_rng(0)
    alpha = rng.random((64, 3)).astype(np.float32)
    alpha[:8] = [[.4, .4, .2], [.2, .4, .4], [.4, .2, .4], [1 / 3, 1 / 3, 1 / 3], [.5, .3, .2], [.2, .5, .3],
                 [.2, .3, .5], [.3, .3, .3]]
    assert (vorta.vorta_route_select(alpha) == vo.hard_route(alpha)).all()
    assert list(vorta.vorta_route_select(alpha[:8])) == [0, 0, 0, 0, 0, 1, 2, 0]


def test_router_gates_are_softmax_of_the_projection():
    """Eq. 3 through the C ABI against the oracle, plus what the mathematics fixes: rows sum to 1,
    a zero embedding gives uniform gates, adding the same vector to the three columns of W_R
    changes nothing, and scaling one column up makes its branch win Eq. 4."""
    rng = np.random.default_rng(3)
    heads, d_t = 40, 256
    T = rng.standard_normal(d_t).astype(np.float32)
    W = (0.1 * rng.standard_normal((heads, d_t, 3))).astype(np.float32)
    got = vorta.vorta_router_gates(T, W)
    want = vo.router_gates(T, W)
    assert got.shape == (heads, 3) and np.abs(got - want).max() < 2e-7
    assert np.abs(got.sum(1) - 1).max() < 1e-6
    assert np.allclose(vorta.vorta_router_gates(np.zeros(d_t, np.float32), W), 1 / 3, atol=1e-7)
    shift = rng.standard_normal((heads, d_t, 1)).astype(np.float32)
    assert np.abs(vorta.vorta_router_gates(T, W + shift) - got).max() < 1e-5
    W2 = W.copy()
    W2[:, :, 2] = 3.0 * T[None, :]            # core-set logit = 3 |T|^2 for every head
    assert (vorta.vorta_route_select(vorta.vorta_router_gates(T, W2)) == 2).all()
    with pytest.raises(vorta.VortaError) as e:
        vorta.vorta_router_gates(np.zeros(0, np.float32), np.zeros((2, 0, 3), np.float32))
    assert e.value.code == -1


def test_bad_descriptions_are_rejected():
    ok = dict(grid=(4, 8, 8), heads=2, head_dim=128, dtype="bf16", tile=(2, 4, 4), window=(3, 3, 3))
    vorta.vorta_plan_create(**ok)
    vorta.vorta_plan_create(**{**ok, "tile": (3, 4, 4)})      # a tile that does not divide the grid is clipped
    for bad, code in ((dict(tile=(0, 4, 4)), -2), (dict(window=(0, 1, 1)), -2), (dict(head_dim=96), -2),
                      (dict(heads=0), -2), (dict(heads=129), -2), (dict(dtype=7), -3), (dict(layout=5), -1),
                      (dict(bucket=(5, 5, 5)), -2), (dict(keep_num=3, keep_den=2), -2),
                      (dict(keep_num=0), -2), (dict(grid=(0, 8, 8)), -2),
                      (dict(rope_dims=(3, 0, 0)), -2), (dict(rope_dims=(64, 64, 2)), -2), (dict(rope_dims=(-2, 0, 0)), -2),
                      (dict(grid=(512, 256, 256), heads=64, layout=0), -2)):     # 2^25 rows x 8192 elements
        with pytest.raises(vorta.VortaError) as e:
            vorta.vorta_plan_create(**{**ok, **bad})
        assert e.value.code == code, bad


def test_workspace_layout_is_aligned_and_ordered():
    cfg = get_config("hunyuan720p")
    plan = vorta.plan_for(cfg)
    routes = make_routes(cfg).numpy()
    off = vorta.vorta_workspace_layout(plan, routes)
    total = vorta.vorta_workspace_bytes(plan, routes)
    assert off[0] == 0 and all(o % 256 == 0 for o in off) and off == sorted(off)
    row = 128 * 2
    assert off[1] - off[0] == 0 and off[4] == 0      # bf16: no tile-ordered copies in the layer call
    assert off[5] - off[4] == 10 * plan.n_core_tokens * row
    assert off[9] - off[8] >= 10 * plan.n_core * 4
    assert total >= off[9] + 10 * plan.n_video * 4
    cfg32 = get_config("tiny")                        # fp32: four tile-ordered buffers per window head
    plan32 = vorta.plan_for(cfg32)
    off32 = vorta.vorta_workspace_layout(plan32, np.array([1, 1], dtype=np.uint8))
    assert off32[1] - off32[0] == 2 * plan32.n_tokens * 64 * 4


def test_tensor_arguments_are_checked_before_the_c_call():
    """The wrappers reject tensors that do not fit the plan -- here with CPU tensors, which fail
    the first check; the shape, dtype and device checks run on the GPU machine."""
    import torch
    cfg = get_config("tiny")
    plan = vorta.plan_for(cfg)
    x = torch.zeros(plan.user_shape())
    for call in (lambda: vorta.vorta_routed_attention_layer(plan, x, x, x, [0, 0]),
                 lambda: vorta.vorta_soft_mixture_layer(plan, x, x, x, np.full((2, 3), 1 / 3)),
                 lambda: vorta.vorta_bcs_build_index(plan, x, [2, 2]),
                 lambda: vorta.vorta_reorder_to_tiles(plan, x, [1, 1])):
        with pytest.raises(vorta.VortaError) as e:
            call()
        assert e.value.code == -1
    with pytest.raises(vorta.VortaError) as e:
        vorta.vorta_soft_mixture_layer(plan, x, x, x, np.full((3, 3), 1 / 3))      # gates for 3 heads, plan has 2
    assert e.value.code == -1 and "alpha" in str(e.value)


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """vorta_host.cpp is plain C++: build it with -fsanitize=address,undefined together with a
    driver that walks every host entry point over ordinary, clipped, oversized and rejected
    descriptions, and run it.  Any report makes the driver exit non-zero."""
    import shutil
    import subprocess
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host compiler")
    csrc = os.path.join(ROOT, "paper_2505_18809_amd", "csrc")
    exe = str(tmp_path / "host_sanitized")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(csrc, "vorta_host.cpp"),
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    run = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-3000:])
    assert "host entry points clean" in run.stdout
