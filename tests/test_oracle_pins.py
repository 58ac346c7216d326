"""Pins for the CPU oracle: each check ties an oracle function to something
other than itself -- hand-worked fixtures, closed forms, brute force written
out in scalar Python, library routines for the special cases that reduce to
them.  No GPU, no HIP library."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import vorta_oracle as vo
from synth_inputs import CONFIGS, get_config, make_qkv
from helpers import f64, smooth_field, spec_of

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_mask_fixture(name):
    out, cur = {}, None
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            out[cur] = []
        else:
            out[cur].append([c == "1" for c in line])
    return {k: np.array(v, dtype=bool) for k, v in out.items()}


# ----------------------------------------------------------------- Eq. 2 ---

def scalar_attention(Q, K, V, scale, keys_of_row=None):
    """Softmax attention with nothing but Python floats."""
    n, d = len(Q), len(V[0])
    out = [[0.0] * d for _ in range(n)]
    for i in range(n):
        keys = range(len(K)) if keys_of_row is None else keys_of_row(i)
        s = [scale * sum(a * b for a, b in zip(Q[i], K[j])) for j in keys]
        m = max(s)
        e = [math.exp(x - m) for x in s]
        z = sum(e)
        for w, j in zip(e, keys):
            for c in range(d):
                out[i][c] += (w / z) * V[j][c]
    return np.array(out)


def test_full_attention_matches_scalar_python():
    rng = np.random.default_rng(0)
    Q, K, V = rng.standard_normal((3, 37, 8))
    spec = vo.LayerSpec(grid=(1, 1, 37), tile=(1, 1, 37), window=(1, 1, 1))
    got = vo.full_attention(Q, K, V, spec)
    want = scalar_attention(Q.tolist(), K.tolist(), V.tolist(), 1 / math.sqrt(8))
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_full_attention_matches_library_sdpa():
    rng = np.random.default_rng(1)
    Q, K, V = rng.standard_normal((3, 200, 16))
    spec = vo.LayerSpec(grid=(2, 10, 10), tile=(1, 5, 5), window=(1, 1, 1))
    got = vo.full_attention(Q, K, V, spec)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0].numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    Q, K, V = rng.standard_normal((3, 50, 4))
    # zero scale: uniform weights -> every row is the mean of V
    spec0 = vo.LayerSpec(grid=(1, 5, 10), tile=(1, 5, 10), window=(1, 1, 1), scale=0.0)
    np.testing.assert_allclose(vo.full_attention(Q, K, V, spec0),
                               np.broadcast_to(V.mean(0), V.shape), atol=1e-14)
    # two keys: weights are a logistic function of the score difference
    q = np.array([[1.0, 2.0]]); k = np.array([[0.5, -1.0], [2.0, 0.25]]); v = np.array([[1.0, 0.0], [0.0, 1.0]])
    s = (q @ k.T)[0] * 0.7
    w1 = 1 / (1 + math.exp(s[0] - s[1]))
    np.testing.assert_allclose(vo.attention_rows(q, k, v, 0.7), [[1 - w1, w1]], atol=1e-15)
    # a key that matches overwhelmingly -> its value row
    big = vo.attention_rows(np.array([[50.0, 0.0]]), np.array([[1.0, 0], [-1.0, 0]]),
                            np.array([[3.0], [7.0]]), 1.0)
    np.testing.assert_allclose(big, [[3.0]], atol=1e-12)
    # rows of P sum to one
    P = vo.softmax_rows(rng.standard_normal((9, 33)) * 5)
    assert np.abs(P.sum(1) - 1).max() < 1e-12 and (P >= 0).all()
    # permuting keys and values together changes nothing; permuting only V does
    perm = rng.permutation(50)
    spec = vo.LayerSpec(grid=(1, 5, 10), tile=(1, 5, 10), window=(1, 1, 1))
    base = vo.full_attention(Q, K, V, spec)
    np.testing.assert_allclose(vo.full_attention(Q, K[perm], V[perm], spec), base, atol=1e-13)
    assert np.abs(vo.full_attention(Q, K, V[perm], spec) - base).max() > 1e-3


@pytest.mark.parametrize("route", [0, 1, 2])
def test_constant_values_give_constant_output(route):
    rng = np.random.default_rng(3)
    grid = (4, 6, 6)
    Q, K = (smooth_field(rng, grid, 8) for _ in range(2))
    V = np.tile(np.array([[1.5, -2.0, 0.25, 4.0, 0, 1, 2, 3]]), (Q.shape[0], 1))
    spec = vo.LayerSpec(grid=grid, tile=(2, 2, 2), window=(1, 3, 1))
    out = vo.head_attention(route, Q, K, V, spec)
    np.testing.assert_allclose(out, V, atol=1e-13)


# ------------------------------------------------------------ Algorithm 1 ---

@pytest.mark.parametrize("name,grid,tile,window", [
    ("sta_mask_1x1x8_tile2_win3.txt", (1, 1, 8), (1, 1, 2), (1, 1, 3)),
    ("sta_mask_2x2x4_tile1x1x2_win1.txt", (2, 2, 4), (1, 1, 2), (1, 1, 1)),
    ("sta_mask_3x1x2_tile1x1x1_win3x1x1.txt", (3, 1, 2), (1, 1, 1), (3, 1, 1)),
    ("sta_mask_1x1x14_tile2_win3_block.txt", (1, 1, 14), (1, 1, 2), (1, 1, 3)),
    ("sta_mask_2x1x5_tile1_win2x1x2_block.txt", (2, 1, 5), (1, 1, 1), (2, 1, 2)),
])
def test_mask_hand_worked_fixtures(name, grid, tile, window):
    for mode, want in read_mask_fixture(name).items():
        got = vo.sta_mask_dense(grid, tile, window, mode)
        assert (got == want).all(), (name, mode)
        rows = np.stack([vo.sta_mask_row(i, grid, tile, window, mode) for i in range(len(want))])
        assert (rows == want).all()
        assert all(vo.sta_mask_entry(i, j, grid, tile, window, mode) == want[i, j]
                   for i in range(len(want)) for j in range(len(want)))


def scalar_mask(grid, tile, window, mode):
    """Algorithm 1 evaluated entry by entry with Python integers, the centre rule written out
    again here: a check of the oracle's vectorised forms that shares none of their code."""
    F, H, W = grid
    L = F * H * W
    n = [-(-g // t) for g, t in zip(grid, tile)]
    def tile_of(i):
        return (i // (H * W) // tile[0], i // W % H // tile[1], i % W // tile[2])
    def centre(q, a):
        w = window[a]
        if mode == "identity":
            return q
        if mode == "block":
            return q - q % w + w // 2
        return sorted((w // 2, q, max(n[a] - 1 - w // 2, w // 2)))[1]      # the middle one = q clamped
    M = np.zeros((L, L), dtype=bool)
    for i in range(L):
        c = [centre(tile_of(i)[a], a) for a in range(3)]
        for j in range(L):
            k = tile_of(j)
            M[i, j] = all(2 * abs(c[a] - k[a]) <= window[a] for a in range(3))
    return M


@pytest.mark.parametrize("mode", ["clamp", "identity", "block"])
@pytest.mark.parametrize("grid,tile,window", [((4, 6, 6), (2, 2, 3), (3, 1, 3)), ((3, 5, 7), (1, 2, 3), (2, 3, 5)),
                                              ((2, 4, 9), (2, 1, 2), (1, 2, 3)), ((5, 7, 6), (2, 3, 4), (3, 3, 3))])
def test_mask_forms_equal_a_scalar_evaluation(grid, tile, window, mode):
    want = scalar_mask(grid, tile, window, mode)
    assert (vo.sta_mask_dense(grid, tile, window, mode) == want).all()
    for i in range(0, want.shape[0], 5):
        assert (vo.sta_mask_row(i, grid, tile, window, mode) == want[i]).all()
        assert all(vo.sta_mask_entry(i, j, grid, tile, window, mode) == want[i, j] for j in range(0, want.shape[1], 3))


@pytest.mark.parametrize("window", [(1, 1, 1), (3, 3, 3), (1, 3, 5), (5, 1, 3), (2, 4, 2)])
def test_mask_row_form_equals_double_loop_and_invariants(window):
    grid, tile = (4, 6, 6), (2, 2, 3)
    n = vo.tile_grid(grid, tile)                      # (2, 3, 2)
    M = vo.sta_mask_dense(grid, tile, window)
    L = M.shape[0]
    for i in range(L):
        assert (vo.sta_mask_row(i, grid, tile, window) == M[i]).all()
    # block-wise dense (section 3.2): constant over (query tile) x (key tile) blocks
    tid = np.array([np.ravel_multi_index(vo.get_tile_id_3d(i, grid, tile), n) for i in range(L)])
    for a in range(n[0] * n[1] * n[2]):
        for b in range(n[0] * n[1] * n[2]):
            blk = M[np.ix_(tid == a, tid == b)]
            assert blk.all() or not blk.any()
    # clamped windows: every query sees prod(min(2*floor(w/2)+1, n)) tiles
    per_axis = [min(2 * (w // 2) + 1, nd) for w, nd in zip(window, n)]
    assert (M.sum(1) == np.prod(per_axis) * np.prod(tile)).all()
    # a token always sees its own tile
    assert M[np.arange(L), np.arange(L)].all()


@pytest.mark.parametrize("window", [(1, 1, 1), (3, 3, 3), (1, 3, 5)])
def test_mask_on_grids_the_tile_does_not_divide(window):
    """Edge tiles are clipped: Algorithm 1's tile id is the integer division of the coordinate,
    so the last tile of an axis just has fewer tokens.  Row form against the double loop, and
    the key count of every row against a count written out per axis: the tiles [lo, hi] of the
    (clamped) window cover coordinates [lo t, min(G, (hi + 1) t))."""
    grid, tile = (5, 7, 6), (2, 3, 4)
    n = vo.tile_grid(grid, tile)
    assert n == (3, 3, 2)
    M = vo.sta_mask_dense(grid, tile, window)
    L = M.shape[0]
    for i in range(L):
        assert (vo.sta_mask_row(i, grid, tile, window) == M[i]).all()
        q = vo.get_tile_id_3d(i, grid, tile)
        count = 1
        for a in range(3):
            half = window[a] // 2
            c = min(max(q[a], half), max(n[a] - 1 - half, half))
            lo, hi = max(c - half, 0), min(c + half, n[a] - 1)
            count *= min(grid[a], (hi + 1) * tile[a]) - lo * tile[a]
        assert M[i].sum() == count
    assert M[np.arange(L), np.arange(L)].all()
    # still block-wise dense over (query tile) x (key tile) blocks, ragged ones included
    tid = np.array([np.ravel_multi_index(vo.get_tile_id_3d(i, grid, tile), n) for i in range(L)])
    sizes = np.bincount(tid)
    for t_id, size in enumerate(sizes):                 # a tile holds the product of its clipped extents
        idx = np.unravel_index(t_id, n)
        assert size == np.prod([min(tile[a], grid[a] - idx[a] * tile[a]) for a in range(3)])
    for a in range(len(sizes)):
        for b in range(len(sizes)):
            blk = M[np.ix_(tid == a, tid == b)]
            assert blk.all() or not blk.any()


def test_mask_covers_everything_when_window_spans_grid():
    grid, tile = (4, 6, 6), (2, 2, 3)
    n = vo.tile_grid(grid, tile)
    for mode in ("clamp", "identity"):
        w = tuple(2 * nd - 1 for nd in n)
        assert vo.sta_mask_dense(grid, tile, w, mode).all()
    # block reading: one block per axis once w >= n, and its middle tile sees the whole axis
    assert vo.sta_mask_dense(grid, tile, tuple(nd + (nd + 1) % 2 for nd in n), "block").all()
    # the Tiny benchmark layer: 2x2x2 tiles under a 3x3x3 window is dense
    tiny = get_config("tiny")
    assert vo.tile_grid(tiny.grid, tiny.tile) == (2, 2, 2)
    assert all(vo.sta_mask_row(i, tiny.grid, tiny.tile, tiny.window).all() for i in range(0, 256, 17))
    # interior tiles: both centre rules agree
    g, t, w = (1, 1, 14), (1, 1, 2), (1, 1, 3)
    a, b = vo.sta_mask_dense(g, t, w, "clamp"), vo.sta_mask_dense(g, t, w, "identity")
    assert (a[2:12] == b[2:12]).all() and not (a[:2] == b[:2]).all()


def test_window_route_equals_full_when_mask_is_dense_and_scalar_brute_force_otherwise():
    rng = np.random.default_rng(4)
    grid = (2, 4, 4)
    Q, K, V = (smooth_field(rng, grid, 6) for _ in range(3))
    dense = vo.LayerSpec(grid=grid, tile=(1, 2, 2), window=(3, 3, 3))
    assert vo.sta_mask_dense(grid, (1, 2, 2), (3, 3, 3)).all()
    np.testing.assert_allclose(vo.window_attention(Q, K, V, dense), vo.full_attention(Q, K, V, dense),
                               atol=1e-12)
    sparse = vo.LayerSpec(grid=grid, tile=(1, 2, 2), window=(1, 1, 1))
    M = vo.sta_mask_dense(grid, sparse.tile, sparse.window)
    want = scalar_attention(Q.tolist(), K.tolist(), V.tolist(), 1 / math.sqrt(6),
                            keys_of_row=lambda i: [j for j in range(32) if M[i, j]])
    got = vo.window_attention(Q, K, V, sparse)
    np.testing.assert_allclose(got, want, atol=1e-13)
    assert np.abs(got - vo.full_attention(Q, K, V, sparse)).max() > 1e-3
    # rows argument picks rows of the same result
    np.testing.assert_allclose(vo.window_attention(Q, K, V, sparse, rows=[5, 31, 0]), want[[5, 31, 0]],
                               atol=1e-13)


def test_window_route_text_tokens():
    rng = np.random.default_rng(5)
    grid, n_text = (2, 2, 4), 3
    L = 16
    Q, K, V = rng.standard_normal((3, L + n_text, 4))
    spec = vo.LayerSpec(grid=grid, tile=(1, 1, 2), window=(1, 1, 1), n_text=n_text)
    M = vo.sta_mask_dense(grid, spec.tile, spec.window)
    def keys(i):
        if i >= L:
            return list(range(L + n_text))
        return [j for j in range(L) if M[i, j]] + list(range(L, L + n_text))
    want = scalar_attention(Q.tolist(), K.tolist(), V.tolist(), 0.5, keys_of_row=keys)
    np.testing.assert_allclose(vo.window_attention(Q, K, V, spec), want, atol=1e-13)


# -------------------------------------------------------------------- BCS ---

def test_bcs_fig3_counts_and_centre():
    for line in open(os.path.join(GOLDEN, "bcs_fig3.txt")):
        if line.startswith("#") or not line.strip():
            continue
        bf, bh, bw, num, den, centre, k = map(int, line.split())
        buckets = list(vo.bcs_buckets((bf, bh, bw), (bf, bh, bw)))
        assert len(buckets) == 1
        idx, c = buckets[0]
        assert c == centre and list(idx) == list(range(bf * bh * bw))
        B = bf * bh * bw
        assert vo.bcs_prune_count(B, num, den) == k
        # the selection itself keeps B - k tokens and sends exactly k others to the centre's slot
        feat = np.random.default_rng(B + num).standard_normal((B, 6))
        keep_idx, assign, _ = vo.bcs_select(feat, (bf, bh, bw), (bf, bh, bw), num, den)
        assert len(keep_idx) == B - k and centre in keep_idx
        assert int((assign == assign[centre]).sum()) == k + 1


@pytest.mark.parametrize("num,den", [(1, 4), (1, 3), (1, 2), (2, 3), (3, 4)])
def test_core_set_length_is_the_kept_share_of_the_sequence(num, den):
    """r_core is the share of the sequence that stays in the core-set (section 4.3: at 50 % the
    core-set is half the original length, and larger ratios cost more computation): on a grid of
    whole 12-token buckets L_c = r L, and a larger r keeps a superset of a smaller one's tokens."""
    grid, bucket = (4, 6, 6), (2, 3, 2)
    L = 4 * 6 * 6
    feat = smooth_field(np.random.default_rng(21), grid, 6)
    keep_idx, assign, _ = vo.bcs_select(feat, grid, bucket, num, den)
    assert len(keep_idx) * den == L * num
    assert len(set(assign)) == len(keep_idx)
    more, _, _ = vo.bcs_select(feat, grid, bucket, min(num + 1, den), den)
    assert set(keep_idx) <= set(more)


def test_bcs_buckets_partition_the_grid_and_clip_at_border():
    grid, bucket = (5, 8, 7), (2, 3, 2)
    seen = np.zeros(5 * 8 * 7, dtype=int)
    shapes = set()
    for idx, c in vo.bcs_buckets(grid, bucket):
        seen[idx] += 1
        coords = np.array([vo.token_coord(int(i), grid) for i in idx])
        ext = coords.max(0) - coords.min(0) + 1
        shapes.add(tuple(ext))
        assert len(idx) == ext.prod() and (ext <= bucket).all()
        assert (coords.min(0) % np.array(bucket) == 0).all()             # origin aligned
        assert tuple(coords[c] - coords.min(0)) == tuple(ext // 2)       # centre = floor(b'/2)
        assert list(idx) == sorted(idx)                                  # local raster order
    assert (seen == 1).all()
    assert (1, 2, 1) in shapes and (2, 3, 2) in shapes


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_bcs_half_ratio_halves_every_benchmark_grid(cfg):
    """Core-set ratio 0.5 (appendix) keeps exactly half the tokens on all five
    grids, so attention cost falls to a quarter (introduction)."""
    kept = sum(len(idx) - vo.bcs_prune_count(len(idx), cfg.keep_num, cfg.keep_den)
               for idx, _ in vo.bcs_buckets(cfg.grid, cfg.bucket))
    assert 2 * kept == cfg.n_video


def test_bcs_similarity_count_is_linear(monkeypatch):
    """L/(thw) buckets x (thw - 1) similarities (appendix complexity paragraph)."""
    calls = []
    real = vo.cosine_to_centre
    monkeypatch.setattr(vo, "cosine_to_centre", lambda a, b: calls.append(1) or real(a, b))
    grid = (4, 6, 6)
    feat = np.random.default_rng(6).standard_normal((144, 5))
    vo.bcs_select(feat, grid, (2, 3, 2))
    assert len(calls) == 144 - 144 // 12


def test_bcs_prunes_the_near_copies_of_the_centre():
    rng = np.random.default_rng(7)
    grid = bucket = (2, 3, 2)
    feat = rng.standard_normal((12, 16))
    centre = 9
    near = [0, 3, 4, 7, 10, 11]
    for j in near:
        feat[j] = feat[centre] * rng.uniform(0.5, 2.0) + 0.01 * rng.standard_normal(16)
    keep_idx, assign, gap = vo.bcs_select(feat, grid, bucket)
    assert sorted(keep_idx) == sorted(set(range(12)) - set(near))
    assert list(keep_idx) == sorted(keep_idx)                      # slots in local raster order
    for j in range(12):
        want = centre if j in near else j
        assert keep_idx[assign[j]] == want
    assert gap > 0.1
    # scaling a token does not change a cosine; flipping its sign does
    feat2 = feat.copy(); feat2[near[0]] *= -1
    k2, _, _ = vo.bcs_select(feat2, grid, bucket)
    assert near[0] in k2


def test_bcs_tie_break_prunes_smaller_index_first():
    feat = np.ones((12, 4))                                        # all cosines equal
    keep_idx, assign, gap = vo.bcs_select(feat, (2, 3, 2), (2, 3, 2))
    assert list(keep_idx) == [6, 7, 8, 9, 10, 11] and gap == 0.0   # 0..5 pruned into centre 9
    assert list(assign) == [3, 3, 3, 3, 3, 3, 0, 1, 2, 3, 4, 5]
    z = np.zeros((12, 4)); z[9] = 1                                # zero-norm tokens: cosine 0
    assert list(vo.bcs_select(z, (2, 3, 2), (2, 3, 2))[0]) == [6, 7, 8, 9, 10, 11]


def test_bcs_identity_cases_reduce_core_set_route_to_full_attention():
    rng = np.random.default_rng(8)
    grid = (3, 4, 5)
    Q, K, V = (smooth_field(rng, grid, 8) for _ in range(3))
    for kw in (dict(keep_num=1, keep_den=1), dict(bucket=(1, 1, 1))):
        spec = vo.LayerSpec(grid=grid, tile=(1, 1, 1), window=(1, 1, 1), **kw)
        keep_idx, assign, _ = vo.bcs_select(K, grid, spec.bucket, spec.keep_num, spec.keep_den)
        # nothing pruned: the core-set is all tokens (bucket-major order; the identity for
        # one-token buckets) and every token reads its own slot
        assert sorted(keep_idx) == list(range(60)) and list(keep_idx[assign]) == list(range(60))
        if spec.bucket == (1, 1, 1):
            assert list(keep_idx) == list(range(60))
        np.testing.assert_allclose(vo.coreset_attention(Q, K, V, spec), vo.full_attention(Q, K, V, spec),
                                   atol=1e-12)


def test_bcs_pool_conserves_mass_and_unpool_inverts_on_kept_tokens():
    rng = np.random.default_rng(9)
    grid = (5, 6, 7)
    X = smooth_field(rng, grid, 6)
    keep_idx, assign, _ = vo.bcs_select(X, grid, (2, 3, 2))
    Xc = vo.bcs_pool(X, keep_idx, assign)
    size = np.bincount(assign, minlength=len(keep_idx))
    np.testing.assert_allclose((size[:, None] * Xc).sum(0), X.sum(0), atol=1e-10)
    singles = size == 1
    np.testing.assert_array_equal(Xc[singles], X[keep_idx[singles]])          # kept tokens untouched
    assert (assign[keep_idx] == np.arange(len(keep_idx))).all()               # a kept token owns its slot
    np.testing.assert_array_equal(vo.bcs_unpool(Xc, assign)[keep_idx], Xc)


@pytest.mark.parametrize("axis,bucket", [(0, (2, 1, 1)), (1, (1, 2, 1)), (2, (1, 1, 2))])
def test_bcs_with_two_token_buckets_is_average_pooling(axis, bucket):
    """Bucket of two at ratio 0.5: the one non-centre token is always pruned, so
    pool() is 2x average pooling along that axis (the ablation's AP variants,
    section 4.3) and unpool() is nearest-neighbour upsampling."""
    rng = np.random.default_rng(10)
    grid = (4, 6, 8)
    X = rng.standard_normal((4 * 6 * 8, 3))
    keep_idx, assign, _ = vo.bcs_select(X, grid, bucket)
    Xc = vo.bcs_pool(X, keep_idx, assign)
    vol = torch.from_numpy(X.reshape(*grid, 3)).permute(3, 0, 1, 2)[None]
    pooled = torch.nn.functional.avg_pool3d(vol, kernel_size=bucket)
    np.testing.assert_allclose(Xc, pooled[0].permute(1, 2, 3, 0).reshape(-1, 3).numpy(), atol=1e-14)
    up = pooled.repeat_interleave(2, dim=2 + axis)[0].permute(1, 2, 3, 0).reshape(-1, 3).numpy()
    np.testing.assert_allclose(vo.bcs_unpool(Xc, assign), up, atol=1e-14)


def scalar_coreset(Q, K, V, grid, bucket, scale, n_text=0, keep=(1, 2)):
    """Core-set route re-derived with Python scalars only, from section 3.2.  keep = r_core as a
    fraction: of a bucket's B tokens, B - floor(B (1 - r)) stay (never fewer than the centre)."""
    F, H, W = grid
    L, d = F * H * W, len(Q[0])
    dot = lambda a, b: sum(x * y for x, y in zip(a, b))
    groups = []                                     # (members, representative token or None)
    for f0 in range(0, F, bucket[0]):
        for h0 in range(0, H, bucket[1]):
            for w0 in range(0, W, bucket[2]):
                fs = range(f0, min(f0 + bucket[0], F)); hs = range(h0, min(h0 + bucket[1], H))
                ws = range(w0, min(w0 + bucket[2], W))
                toks = [(f * H + h) * W + w for f in fs for h in hs for w in ws]
                cf, ch, cw = fs[len(fs) // 2], hs[len(hs) // 2], ws[len(ws) // 2]
                c = (cf * H + ch) * W + cw
                sims = []
                for t in toks:
                    if t != c:
                        den = math.sqrt(dot(K[c], K[c]) * dot(K[t], K[t]))
                        sims.append((-(dot(K[c], K[t]) / den if den else 0.0), t))
                n_stay = max(1, len(toks) - (len(toks) * (keep[1] - keep[0])) // keep[1])
                k = len(toks) - n_stay
                dropped = [t for _, t in sorted(sims)[:k]]
                for t in toks:
                    if t not in dropped:
                        groups.append([t] + (dropped if t == c else []))
    groups += [[L + t] for t in range(n_text)]
    mean = lambda X, g: [sum(X[t][c] for t in g) / len(g) for c in range(d)]
    Qc, Kc, Vc = ([mean(X, g) for g in groups] for X in (Q, K, V))
    Oc = scalar_attention(Qc, Kc, Vc, scale)
    out = np.zeros((L + n_text, d))
    for s, g in enumerate(groups):
        out[g] = Oc[s]
    return out


@pytest.mark.parametrize("grid,n_text,keep", [((2, 3, 4), 0, (1, 2)), ((3, 4, 3), 2, (1, 2)),
                                              ((2, 3, 4), 1, (1, 4)), ((3, 4, 3), 0, (3, 4)), ((2, 6, 2), 2, (2, 3))])
def test_coreset_route_matches_scalar_rederivation(grid, n_text, keep):
    rng = np.random.default_rng(11)
    L = grid[0] * grid[1] * grid[2]
    Q, K, V = (np.concatenate([smooth_field(rng, grid, 5), rng.standard_normal((n_text, 5))]) for _ in range(3))
    spec = vo.LayerSpec(grid=grid, tile=(1, 1, 1), window=(1, 1, 1), n_text=n_text, scale=0.4,
                        keep_num=keep[0], keep_den=keep[1])
    want = scalar_coreset(Q.tolist(), K.tolist(), V.tolist(), grid, (2, 3, 2), 0.4, n_text, keep)
    got = vo.coreset_attention(Q, K, V, spec)
    np.testing.assert_allclose(got, want, atol=1e-13)
    np.testing.assert_allclose(vo.coreset_attention(Q, K, V, spec, rows=[L + n_text - 1, 3, 0]),
                               want[[L + n_text - 1, 3, 0]], atol=1e-13)
    assert np.abs(got - vo.full_attention(Q, K, V, spec)).max() > 1e-3


# ------------------------------------------------------------------- RoPE ---

def complex_rope(X, coords, rope_dims, theta):
    """The same rotation written with complex numbers: channel pairs are complex values that are
    multiplied by exp(i * position * rate).  Python scalars only."""
    out = [list(map(float, row)) for row in X]
    for r, (row, pos) in enumerate(zip(X, coords)):
        start = 0
        for axis, span in enumerate(rope_dims):
            for i in range(span // 2):
                z = complex(row[start + 2 * i], row[start + 2 * i + 1])
                z *= complex(math.cos(pos[axis] * theta ** (-2 * i / span)), math.sin(pos[axis] * theta ** (-2 * i / span)))
                out[r][start + 2 * i], out[r][start + 2 * i + 1] = z.real, z.imag
            start += span
    return np.array(out)


def test_rope_hand_computed_turns_and_what_it_leaves_alone():
    # one pair, span 2: the rate is theta^0 = 1, so position p turns (1, 0) by p radians
    X = np.array([[1.0, 0.0, 7.0], [0.0, 2.0, 7.0]])
    Y = vo.rope_rotate(X, [[3, 0, 0], [3, 0, 0]], (2, 0, 0), 10000.0)
    np.testing.assert_allclose(Y, [[math.cos(3), math.sin(3), 7.0], [-2 * math.sin(3), 2 * math.cos(3), 7.0]], atol=1e-15)
    # span 4 at theta = 10000: pair 0 turns by p, pair 1 by p / 100; the H axis uses the row index
    X = np.array([[1.0, 0.0, 1.0, 0.0, 5.0, 6.0]])
    Y = vo.rope_rotate(X, [[9, 50, 2]], (0, 4, 0), 10000.0)
    np.testing.assert_allclose(Y, [[math.cos(50), math.sin(50), math.cos(0.5), math.sin(0.5), 5.0, 6.0]], atol=1e-14)
    # the origin is the identity; channels past the three spans never move
    X = np.random.default_rng(30).standard_normal((4, 12))
    np.testing.assert_array_equal(vo.rope_rotate(X, np.zeros((4, 3), int), (4, 2, 4)), X)
    Y = vo.rope_rotate(X, [[1, 2, 3]] * 4, (4, 2, 4))
    np.testing.assert_array_equal(Y[:, 10:], X[:, 10:])
    assert np.abs(Y[:, :10] - X[:, :10]).min() > 0
    # moving along one axis only changes that axis' channels
    Z = vo.rope_rotate(X, [[1, 2, 8]] * 4, (4, 2, 4))
    np.testing.assert_array_equal(Z[:, :6], Y[:, :6])
    assert np.abs(Z[:, 6:10] - Y[:, 6:10]).min() > 0


def test_rope_is_a_rotation_that_depends_on_relative_position_only():
    rng = np.random.default_rng(31)
    dims, theta = (4, 6, 6), 100.0
    q, k = rng.standard_normal((2, 1, 20))
    pi, pj, shift = np.array([[3, 7, 2]]), np.array([[1, 4, 9]]), np.array([[5, 11, 6]])
    Rq, Rk = vo.rope_rotate(q, pi, dims, theta), vo.rope_rotate(k, pj, dims, theta)
    # norms of every pair survive
    np.testing.assert_allclose(Rq[0, 0:16:2] ** 2 + Rq[0, 1:16:2] ** 2, q[0, 0:16:2] ** 2 + q[0, 1:16:2] ** 2, atol=1e-13)
    # <R_i q, R_j k> is unchanged when both positions move together, and equals <q, R_(j-i) k>
    moved = vo.rope_rotate(q, pi + shift, dims, theta) @ vo.rope_rotate(k, pj + shift, dims, theta).T
    np.testing.assert_allclose(moved, Rq @ Rk.T, atol=1e-12)
    np.testing.assert_allclose(q @ vo.rope_rotate(k, pj - pi, dims, theta).T, Rq @ Rk.T, atol=1e-12)
    assert abs((vo.rope_rotate(q, pi + shift, dims, theta) @ Rk.T - Rq @ Rk.T).item()) > 1e-3
    # turning by a then by b is turning by a + b
    twice = vo.rope_rotate(vo.rope_rotate(q, pi, dims, theta), shift, dims, theta)
    np.testing.assert_allclose(twice, vo.rope_rotate(q, pi + shift, dims, theta), atol=1e-13)
    # against the complex-number form, scalar Python
    X = rng.standard_normal((6, 20))
    coords = rng.integers(0, 30, (6, 3))
    np.testing.assert_allclose(vo.rope_rotate(X, coords, dims, theta), complex_rope(X.tolist(), coords.tolist(), dims, theta),
                               atol=1e-13)


@pytest.mark.parametrize("n_text", [0, 3])
def test_routes_with_rope_rotate_queries_and_keys_at_the_right_point(n_text):
    """Routes 0 and 1: plain attention on Q and K rotated by their own grid position (text rows
    unrotated).  Route 2: pooling acts before the rotation and a core-set row turns with the
    position of the token that owns its slot -- rebuilt here from pool(), the complex form and
    plain attention."""
    rng = np.random.default_rng(32)
    grid, d = (2, 3, 4), 8
    L = 24
    dims, theta = (2, 2, 4), 50.0
    Q, K, V = (np.concatenate([smooth_field(rng, grid, d), rng.standard_normal((n_text, d))]) for _ in range(3))
    spec = vo.LayerSpec(grid=grid, tile=(1, 3, 2), window=(1, 1, 1), n_text=n_text, scale=0.3, rope_dims=dims, rope_theta=theta)
    plain = vo.LayerSpec(grid=grid, tile=(1, 3, 2), window=(1, 1, 1), n_text=n_text, scale=0.3)
    coords = [list(vo.token_coord(i, grid)) for i in range(L)]
    turn = lambda X, c: np.concatenate([complex_rope(X[:len(c)].tolist(), c, dims, theta), X[len(c):]])
    Qr, Kr = turn(Q, coords), turn(K, coords)
    np.testing.assert_allclose(vo.full_attention(Q, K, V, spec), vo.full_attention(Qr, Kr, V, plain), atol=1e-12)
    np.testing.assert_allclose(vo.window_attention(Q, K, V, spec), vo.window_attention(Qr, Kr, V, plain), atol=1e-12)
    assert np.abs(vo.full_attention(Q, K, V, spec) - vo.full_attention(Q, K, V, plain)).max() > 1e-3
    keep_idx, assign, _ = vo.bcs_select(K[:L], grid, spec.bucket)           # selection sees the un-rotated keys
    slot_coords = [coords[i] for i in keep_idx]
    Qc = np.concatenate([turn(vo.bcs_pool(Q[:L], keep_idx, assign), slot_coords), Q[L:]])
    Kc = np.concatenate([turn(vo.bcs_pool(K[:L], keep_idx, assign), slot_coords), K[L:]])
    Vc = np.concatenate([vo.bcs_pool(V[:L], keep_idx, assign), V[L:]])
    Oc = vo.attention_rows(Qc, Kc, Vc, 0.3)
    want = np.concatenate([Oc[assign], Oc[len(keep_idx):]])
    np.testing.assert_allclose(vo.coreset_attention(Q, K, V, spec), want, atol=1e-12)
    # rotate-then-pool would be something else
    other = vo.coreset_attention(Qr, Kr, V, plain, feat=K)
    assert np.abs(other - want).max() > 1e-3
    # rows= picks rows of the same result
    np.testing.assert_allclose(vo.coreset_attention(Q, K, V, spec, rows=[L + n_text - 1, 0, 5]), want[[L + n_text - 1, 0, 5]],
                               atol=1e-13)


# ---------------------------------------------------------------- routing ---

def test_hard_route_follows_eq4_and_sends_ties_to_full():
    a = np.array([[0.5, 0.3, 0.2], [0.2, 0.5, 0.3], [0.2, 0.3, 0.5],
                  [0.4, 0.4, 0.2], [0.2, 0.4, 0.4], [0.4, 0.2, 0.4], [1 / 3, 1 / 3, 1 / 3]])
    assert list(vo.hard_route(a)) == [0, 1, 2, 0, 0, 0, 0]


def test_router_gates_are_a_softmax_of_a_linear_map():
    rng = np.random.default_rng(12)
    T, W = rng.standard_normal(7), rng.standard_normal((4, 7, 3))
    g = vo.router_gates(T, W)
    assert g.shape == (4, 3) and np.abs(g.sum(1) - 1).max() < 1e-14
    z = [sum(T[i] * W[2, i, k] for i in range(7)) for k in range(3)]
    e = [math.exp(x) for x in z]
    np.testing.assert_allclose(g[2], [x / sum(e) for x in e], atol=1e-14)
    np.testing.assert_allclose(vo.router_gates(np.zeros(7), W), 1 / 3)


def test_layer_dispatches_each_head_by_its_route_and_soft_mixture_blends():
    rng = np.random.default_rng(13)
    grid = (2, 6, 4)
    Q, K, V = (np.stack([smooth_field(rng, grid, 4) for _ in range(3)]) for _ in range(3))
    spec = vo.LayerSpec(grid=grid, tile=(1, 3, 2), window=(1, 1, 1))
    out = vo.routed_attention_layer(Q, K, V, [2, 0, 1], spec)
    np.testing.assert_array_equal(out[0], vo.coreset_attention(Q[0], K[0], V[0], spec))
    np.testing.assert_array_equal(out[1], vo.full_attention(Q[1], K[1], V[1], spec))
    np.testing.assert_array_equal(out[2], vo.window_attention(Q[2], K[2], V[2], spec))
    onehot = np.eye(3)[[2, 0, 1]]
    np.testing.assert_allclose(vo.soft_mixture_layer(Q, K, V, onehot, spec), out, atol=1e-14)
    mix = vo.soft_mixture_layer(Q, K, V, np.full((3, 3), 1 / 3), spec)
    want0 = sum(vo.head_attention(r, Q[0], K[0], V[0], spec) for r in range(3)) / 3
    np.testing.assert_allclose(mix[0], want0, atol=1e-14)


# ------------------------------------------------------- synthetic inputs ---

def test_synthetic_fields_follow_the_recipe():
    from scipy.ndimage import gaussian_filter1d
    from synth_inputs import blur_matrix
    x = np.random.default_rng(14).standard_normal(23)
    np.testing.assert_allclose(blur_matrix(23).numpy() @ x,
                               gaussian_filter1d(x, sigma=2.0, truncate=4.0, mode="reflect"), atol=1e-13)
    np.testing.assert_allclose(blur_matrix(4).numpy() @ x[:4],
                               gaussian_filter1d(x[:4], sigma=2.0, truncate=4.0, mode="reflect"), atol=1e-13)
    cfg = get_config("tiny")
    q, k, v = make_qkv(cfg)
    q2, _, _ = make_qkv(cfg)
    assert q.shape == (2, 256, 64) and q.dtype == torch.float32 and torch.equal(q, q2)
    for t in (q, k, v):
        assert abs(float(t.mean())) < 0.05 and abs(float(t.std()) - 1) < 0.05
    assert not torch.equal(q, k)
    # neighbours along W are correlated, far tokens are not
    kk = f64(k[0]).reshape(4, 8, 8, 64)
    near = np.mean(kk[:, :, :-1] * kk[:, :, 1:]); far = np.mean(kk[:, :, 0] * kk[:, :, 7])
    assert near > 0.5 and abs(far) < 0.35
    q0, _, _ = make_qkv(cfg, layout=0)
    assert q0.shape == (256, 2, 64) and torch.equal(q0.transpose(0, 1), q)


def test_route_vectors():
    from synth_inputs import make_routes
    assert list(make_routes(get_config("single"))) == [0, 0, 1, 1, 1, 2, 2, 2]
    for name, counts in (("wan480p", (8, 16, 16)), ("wan720p", (6, 18, 16)), ("hunyuan720p", (2, 12, 10))):
        r = make_routes(get_config(name))
        assert tuple(int((r == i).sum()) for i in range(3)) == counts
        assert torch.equal(r, make_routes(get_config(name)))
