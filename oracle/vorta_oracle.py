"""CPU oracle for VORTA's routed attention layer (arXiv 2505.18809).

TEST INFRASTRUCTURE ONLY.  Plain NumPy in fp64, written from the paper, slow
on purpose and with no blocking or fusion.  It shares no code with the HIP
library and must never be imported by it; only tests, the smoke check and the
benchmark's cpu_baseline leg call it.

What each function follows:
  full attention ............ Eq. 2 (softmax(Q K^T) V; a 1/sqrt(d) scale is a parameter)
  sliding tile mask ......... Algorithm 1 (appendix "Methodological details")
  core-set attention ........ section 3.2 "Core-set selection": unpool . attn . pool,
                              pool = Bucketed Core-set Selection (Fig. 3, appendix
                              complexity paragraph)
  routing ................... Eq. 3 (gates) and Eq. 4 (hard selection)
  soft mixture .............. Eq. 5
  rotary embedding .......... named in section 3.3 as part of the block, not defined there: the
                              axial 3-D form is a reading (see the section on it below)

Readings taken where the paper is silent (kept in one place so a reader can
check them):
  * tokens are the (F,H,W) grid flattened frame-major; 0-based indices.
  * get_tile_id_3d = per-axis floor(coord / tile); where the tile does not
    divide an axis, the last tile of that axis is clipped to the grid.
  * get_window_center_id clamps the query tile id so the window stays inside
    the tile grid (mode "clamp", the sliding-*tile* behaviour); mode
    "identity" leaves it unchanged (windows truncated at the border); mode
    "block" gives every query tile of a block of w tiles the block's middle
    tile (the 3-D form of section 3.2's tau(i)).
  * similarity = cosine between the bucket's centre token and each other token
    of the bucket, on a caller-chosen feature (the head's keys by default).
  * centre = token at local coordinate floor(b'/2) per axis of the (possibly
    border-clipped) bucket; k = floor(B' * (1 - r)) tokens are pruned (at most
    B' - 1), highest similarity first, ties broken towards the smaller local
    raster index.
  * "merged into the centre" = arithmetic mean of the centre and its pruned
    tokens, applied alike to Q, K and V; kept tokens are unchanged.
  * text tokens follow the video tokens, are never tiled, bucketed or pooled,
    are visible as keys to every query, and as queries see every key of the
    route's key set.

Parity status: every function below is pinned by tests/test_oracle_*.py
against brute force, closed forms or special cases that reduce to textbook
softmax attention / average pooling.  The whole core-set route has no
published numeric example: it is pinned to those special cases and to a
scalar re-derivation on tiny grids, and beyond that is "parity unpinned"
against the authors' own code.  The rotary embedding is pinned by what the
mathematics fixes (norms, dependence on relative position only, composition,
the identity at the origin, a hand-computed 2-D turn); which channels belong to
which axis and how channels pair up is a reading: "parity unpinned" against the
authors' models.
"""
from dataclasses import dataclass
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

ROUTE_FULL, ROUTE_WINDOW, ROUTE_CORESET = 0, 1, 2


@dataclass(frozen=True)
class LayerSpec:
    grid: Tuple[int, int, int]
    tile: Tuple[int, int, int]
    window: Tuple[int, int, int]                 # in tiles, as Algorithm 1 compares tile ids
    bucket: Tuple[int, int, int] = (2, 3, 2)
    keep_num: int = 1                            # r_core = keep_num / keep_den
    keep_den: int = 2
    n_text: int = 0
    scale: Optional[float] = None                # None -> 1/sqrt(head_dim)
    center_mode: str = "clamp"
    rope_dims: Optional[Tuple[int, int, int]] = None   # channels rotated by the F, H, W position; None = no RoPE
    rope_theta: float = 10000.0

    @property
    def n_video(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2]


# --------------------------------------------------------------------------
# token / tile geometry (Algorithm 1)
# --------------------------------------------------------------------------

def token_coord(i: int, grid) -> Tuple[int, int, int]:
    """Frame-major raster index -> (f, h, w)."""
    _, H, W = grid
    return (i // (H * W), (i // W) % H, i % W)


def get_tile_id_3d(i: int, grid, tile) -> Tuple[int, int, int]:
    c = token_coord(i, grid)
    return (c[0] // tile[0], c[1] // tile[1], c[2] // tile[2])


def tile_grid(grid, tile) -> Tuple[int, int, int]:
    """Tiles per axis.  Algorithm 1 assigns tile ids by integer division of the
    token coordinate, whatever the grid: when the tile does not divide an axis
    the last tile of that axis is simply smaller, so there are ceil(G / t) of
    them (the same clipping as for edge buckets)."""
    return tuple(-(-g // t) for g, t in zip(grid, tile))


CENTER_MODES = ("clamp", "identity", "block")


def get_window_center_id(q, n_tiles, window, mode: str = "clamp"):
    """Tile id the window of query tile q is centred on (Algorithm 1 names the function and
    says only that all queries of one window share the centre's tile id).  Three readings:
      clamp     the query tile's id, moved inward so that the window stays inside the tile grid
                (the sliding-tile behaviour section 3.2 adopts); the default
      identity  the query tile's own id (windows cut off at the border)
      block     the tile grid is cut into blocks of w tiles per axis and every query tile of a
                block shares the block's middle tile, floor(q / w) w + floor(w / 2) -- the 3-D
                form of section 3.2's tau(i); the centre of a partial last block may lie past
                the grid, which only means fewer of its key tiles exist."""
    if mode not in CENTER_MODES:
        raise ValueError(mode)
    if mode == "identity":
        return tuple(q)
    if mode == "block":
        return tuple((qd // wd) * wd + wd // 2 for qd, wd in zip(q, window))
    out = []
    for qd, nd, wd in zip(q, n_tiles, window):
        half = wd // 2
        lo, hi = half, max(nd - 1 - half, half)
        out.append(min(max(qd, lo), hi))
    return tuple(out)


def axis_tile_ids(grid, tile):
    """Per axis, the tile id of every token of the flattened grid: three int arrays of length L."""
    F, H, W = grid
    i = np.arange(F * H * W)
    return ((i // (H * W)) // tile[0], ((i // W) % H) // tile[1], (i % W) // tile[2])


def visible_key_tiles(centre, n_tiles, window):
    """Algorithm 1's test per axis: key tile k of axis a is visible from a window centred on
    centre[a] when abs(centre[a] - k) <= window[a] / 2.  Returns three boolean vectors over the
    tile ids of each axis; a key tile is visible when all three of its coordinates are."""
    return tuple(np.abs(c - np.arange(n)) <= w / 2 for c, n, w in zip(centre, n_tiles, window))


def sta_mask_row(i: int, grid, tile, window, mode: str = "clamp") -> np.ndarray:
    """Row i of Algorithm 1's mask M: the keys whose tile is visible from query i's window."""
    n_tiles = tile_grid(grid, tile)
    centre = get_window_center_id(get_tile_id_3d(i, grid, tile), n_tiles, window, mode)
    vis = visible_key_tiles(centre, n_tiles, window)
    kf, kh, kw = axis_tile_ids(grid, tile)
    return vis[0][kf] & vis[1][kh] & vis[2][kw]


def sta_mask_entry(i: int, j: int, grid, tile, window, mode: str = "clamp") -> bool:
    """One entry M[i, j]: is key j's tile inside the window of query i?"""
    n_tiles = tile_grid(grid, tile)
    centre = get_window_center_id(get_tile_id_3d(i, grid, tile), n_tiles, window, mode)
    key_tile = get_tile_id_3d(j, grid, tile)
    return all(abs(c - k) <= w / 2 for c, k, w in zip(centre, key_tile, window))


def sta_mask_dense(grid, tile, window, mode: str = "clamp") -> np.ndarray:
    """The whole L x L mask, built tile block by tile block: the mask is constant over
    (query tile) x (key tile) blocks, so each query tile's visible key tiles are expanded to
    tokens once.  Tiny grids only."""
    n_tiles = tile_grid(grid, tile)
    kf, kh, kw = axis_tile_ids(grid, tile)
    L = len(kf)
    M = np.zeros((L, L), dtype=bool)
    for qf in range(n_tiles[0]):
        for qh in range(n_tiles[1]):
            for qw in range(n_tiles[2]):
                centre = get_window_center_id((qf, qh, qw), n_tiles, window, mode)
                vis = visible_key_tiles(centre, n_tiles, window)
                queries = (kf == qf) & (kh == qh) & (kw == qw)
                M[np.ix_(queries, vis[0][kf] & vis[1][kh] & vis[2][kw])] = True
    return M


# --------------------------------------------------------------------------
# rotary position embedding on the 3-D grid
#
# The paper's block applies RoPE to Q and K and leaves it out of its equations "for clarity"
# (section 3.3, "Inference-time routing strategy"), so the rotation itself is a reading: the
# axial 3-D form video DiTs use.  The first rope_dims[0] channels of a head are rotated by the
# token's frame index, the next rope_dims[1] by its row, the next rope_dims[2] by its column;
# channels beyond their sum and text tokens are left alone.  Inside an axis' span, channels
# (2i, 2i+1) form a pair that is turned by the angle  pos * theta^(-2i / span).
# Core-set branch: pool() acts on the block's input, i.e. before the rotation (pooling commutes
# with the linear projections, not with RoPE); a core-set row is then rotated with the position
# of the token that owns its slot (a merged centre keeps the centre's position).
# --------------------------------------------------------------------------

def rope_angles(positions, span: int, theta: float) -> np.ndarray:
    """[n] integer positions -> [n, span / 2] angles pos * theta^(-2 i / span)."""
    i = np.arange(span // 2, dtype=np.float64)
    return np.asarray(positions, dtype=np.float64)[:, None] * theta ** (-2.0 * i / span)[None, :]


def rope_rotate(X, coords, rope_dims, theta: float = 10000.0) -> np.ndarray:
    """X: [n, d]; coords: [n, 3] integer (f, h, w) of every row.  Returns the rotated copy."""
    X = np.asarray(X, dtype=np.float64)
    coords = np.asarray(coords)
    assert all(s % 2 == 0 and s >= 0 for s in rope_dims) and sum(rope_dims) <= X.shape[1]
    out = X.copy()
    start = 0
    for axis, span in enumerate(rope_dims):
        if span:
            ang = rope_angles(coords[:, axis], span, theta)
            a, b = X[:, start:start + span:2], X[:, start + 1:start + span:2]
            out[:, start:start + span:2] = a * np.cos(ang) - b * np.sin(ang)
            out[:, start + 1:start + span:2] = a * np.sin(ang) + b * np.cos(ang)
        start += span
    return out


def rope_video_rows(X, spec: "LayerSpec", token_ids=None) -> np.ndarray:
    """Rotate the rows of X that belong to video tokens: row r holds token token_ids[r]
    (default r itself); rows past the video tokens (text) are returned unchanged."""
    X = np.asarray(X, dtype=np.float64)
    if spec.rope_dims is None:
        return X
    n = X.shape[0] if token_ids is None else len(token_ids)
    ids = np.arange(min(n, spec.n_video)) if token_ids is None else np.asarray(token_ids, dtype=np.int64)
    coords = np.array([token_coord(int(i), spec.grid) for i in ids]).reshape(-1, 3)
    out = X.copy()
    out[:len(ids)] = rope_rotate(X[:len(ids)], coords, spec.rope_dims, spec.rope_theta)
    return out


# --------------------------------------------------------------------------
# softmax attention (Eq. 2)
# --------------------------------------------------------------------------

def softmax_rows(S: np.ndarray) -> np.ndarray:
    S = S - S.max(axis=-1, keepdims=True)
    P = np.exp(S)
    return P / P.sum(axis=-1, keepdims=True)


def attention_rows(q_rows: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float,
                   chunk: int = 256) -> np.ndarray:
    """softmax(scale * q K^T) V for the given query rows over ALL rows of K, V."""
    q_rows = np.asarray(q_rows, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    out = np.empty((q_rows.shape[0], V.shape[1]), dtype=np.float64)
    for s in range(0, q_rows.shape[0], chunk):
        P = softmax_rows(scale * (q_rows[s:s + chunk] @ K.T))
        out[s:s + chunk] = P @ V
    return out


def _scale(spec: LayerSpec, d: int) -> float:
    return spec.scale if spec.scale is not None else 1.0 / np.sqrt(d)


def _all_rows(n: int, rows) -> np.ndarray:
    return np.arange(n) if rows is None else np.asarray(rows, dtype=np.int64)


def full_attention(Q, K, V, spec: LayerSpec, rows=None) -> np.ndarray:
    """Route 0.  Q, K, V: [N, d] of one head (before RoPE, if the spec has one).  Returns O[rows]."""
    Q = rope_video_rows(Q, spec)
    K = rope_video_rows(K, spec)
    rows = _all_rows(Q.shape[0], rows)
    return attention_rows(Q[rows], K, V, _scale(spec, Q.shape[1]))


def window_attention(Q, K, V, spec: LayerSpec, rows=None) -> np.ndarray:
    """Route 1: softmax attention restricted to Algorithm 1's mask; text
    tokens (if any) are unmasked in both directions."""
    Q = rope_video_rows(Q, spec)
    K = rope_video_rows(K, spec)
    V = np.asarray(V, dtype=np.float64)
    L, N = spec.n_video, Q.shape[0]
    assert N == L + spec.n_text
    rows = _all_rows(N, rows)
    scale = _scale(spec, Q.shape[1])
    out = np.empty((len(rows), V.shape[1]), dtype=np.float64)
    n_tiles = tile_grid(spec.grid, spec.tile)
    cache: Dict[tuple, np.ndarray] = {}          # mask rows repeat within a query tile
    for r, i in enumerate(rows):
        i = int(i)
        if i >= L:
            keys = np.arange(N)
        else:
            key = get_window_center_id(get_tile_id_3d(i, spec.grid, spec.tile), n_tiles,
                                       spec.window, spec.center_mode)
            if key not in cache:
                m = sta_mask_row(i, spec.grid, spec.tile, spec.window, spec.center_mode)
                cache[key] = np.concatenate([np.nonzero(m)[0], np.arange(L, N)])
            keys = cache[key]
        out[r] = attention_rows(Q[i:i + 1], K[keys], V[keys], scale)[0]
    return out


# --------------------------------------------------------------------------
# Bucketed Core-set Selection (section 3.2, Fig. 3)
# --------------------------------------------------------------------------

def bcs_buckets(grid, bucket):
    """Yield (token_indices, centre_pos) per bucket.  Buckets tile the grid
    from the origin, in raster order of bucket coordinates, clipped at the
    border; token_indices are global raster indices in the bucket's local
    raster order; centre_pos indexes into token_indices."""
    F, H, W = grid
    bf, bh, bw = bucket
    for f0 in range(0, F, bf):
        for h0 in range(0, H, bh):
            for w0 in range(0, W, bw):
                df, dh, dw = min(bf, F - f0), min(bh, H - h0), min(bw, W - w0)
                idx = [((f0 + a) * H + (h0 + b)) * W + (w0 + c)
                       for a in range(df) for b in range(dh) for c in range(dw)]
                centre = ((df // 2) * dh + (dh // 2)) * dw + (dw // 2)
                yield np.asarray(idx, dtype=np.int64), centre


def bcs_prune_count(bucket_size: int, keep_num: int, keep_den: int) -> int:
    """k = floor(B' (1 - r)), never pruning the centre itself.  r = keep_num / keep_den is the
    share of the sequence that STAYS (section 4.3: the core-set at r_core = 50 % has half the
    original length, and larger ratios cost more computation)."""
    return min(bucket_size - 1, (bucket_size * (keep_den - keep_num)) // keep_den)


def cosine_to_centre(xc: np.ndarray, xj: np.ndarray) -> float:
    nc, nj = float(xc @ xc), float(xj @ xj)
    if nc == 0.0 or nj == 0.0:
        return 0.0
    return float(xc @ xj) / float(np.sqrt(nc * nj))


def bcs_select(feat, grid, bucket=(2, 3, 2), keep_num=1, keep_den=2):
    """Core-set index for one head.

    feat: [L, d] feature the similarity is taken on.
    Returns keep_idx int32[L_c] (raster index of the token in each core-set
    slot), assign int32[L] (slot each token reads its output from) and the
    smallest gap between a pruned and a kept similarity (inf if no bucket has
    both) -- a guard for the tie-break being the only source of order."""
    feat = np.asarray(feat, dtype=np.float64)
    L = grid[0] * grid[1] * grid[2]
    assert feat.shape[0] == L
    keep_idx = []
    assign = np.full(L, -1, dtype=np.int64)
    min_gap = np.inf
    for idx, c in bcs_buckets(grid, bucket):
        B = len(idx)
        k = bcs_prune_count(B, keep_num, keep_den)
        others = [j for j in range(B) if j != c]
        sims = {j: cosine_to_centre(feat[idx[c]], feat[idx[j]]) for j in others}
        ranked = sorted(others, key=lambda j: (-sims[j], j))
        pruned = set(ranked[:k])
        if 0 < k < len(others):
            min_gap = min(min_gap, sims[ranked[k - 1]] - sims[ranked[k]])
        kept = [j for j in range(B) if j not in pruned]
        base = len(keep_idx)
        slot_of = {j: base + s for s, j in enumerate(kept)}
        keep_idx.extend(int(idx[j]) for j in kept)
        for j in range(B):
            assign[idx[j]] = slot_of[j] if j in slot_of else slot_of[c]
    assert (assign >= 0).all()
    return np.asarray(keep_idx, dtype=np.int32), assign.astype(np.int32), float(min_gap)


def bcs_pool(X, keep_idx, assign) -> np.ndarray:
    """pool(): X_c[slot] = mean of the tokens assigned to that slot -- the slot's
    own token, plus, for a centre, the tokens pruned into it."""
    X = np.asarray(X, dtype=np.float64)
    Xc = np.zeros((len(keep_idx), X.shape[1]), dtype=np.float64)
    cnt = np.zeros(len(keep_idx), dtype=np.int64)
    for i in range(len(assign)):
        Xc[assign[i]] += X[i]
        cnt[assign[i]] += 1
    return Xc / cnt[:, None]


def bcs_unpool(Oc, assign) -> np.ndarray:
    """unpool(): every token reads the output of the slot it was assigned to."""
    return np.asarray(Oc)[np.asarray(assign)]


def coreset_attention(Q, K, V, spec: LayerSpec, rows=None, feat=None, index=None) -> np.ndarray:
    """Route 2: unpool(attn(pool(.))).  feat defaults to the head's keys."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    L, N = spec.n_video, Q.shape[0]
    assert N == L + spec.n_text
    if index is None:
        f = K[:L] if feat is None else np.asarray(feat, dtype=np.float64)[:L]
        index = bcs_select(f, spec.grid, spec.bucket, spec.keep_num, spec.keep_den)
    keep_idx, assign = index[0], index[1]
    Lc = len(keep_idx)
    # pool first (on the un-rotated rows), then rotate each core-set row with its slot owner's position
    Qc = np.concatenate([rope_video_rows(bcs_pool(Q[:L], keep_idx, assign), spec, keep_idx), Q[L:]])
    Kc = np.concatenate([rope_video_rows(bcs_pool(K[:L], keep_idx, assign), spec, keep_idx), K[L:]])
    Vc = np.concatenate([bcs_pool(V[:L], keep_idx, assign), V[L:]])
    # slot every output row reads from: video tokens via assign, text tokens their own
    src = np.concatenate([assign.astype(np.int64), Lc + np.arange(spec.n_text)])
    rows = _all_rows(N, rows)
    need = src[rows]
    uniq, inv = np.unique(need, return_inverse=True)
    Oc = attention_rows(Qc[uniq], Kc, Vc, _scale(spec, Q.shape[1]))
    return Oc[inv]


# --------------------------------------------------------------------------
# routing (Eq. 3-5) and the routed layer
# --------------------------------------------------------------------------

def router_gates(T, W_R) -> np.ndarray:
    """Eq. 3: alpha = softmax(T W_R).  T: [d_t]; W_R: [d_t, 3] or, one router per
    head, [heads, d_t, 3].  Returns [..., 3] = (full, sliding, core-set)."""
    T = np.asarray(T, dtype=np.float64)
    W_R = np.asarray(W_R, dtype=np.float64)
    return softmax_rows(np.einsum("d,...dk->...k", T, W_R))


def hard_route(alpha) -> np.ndarray:
    """Eq. 4: sliding iff a2 beats both others strictly, core-set iff a3 does,
    full otherwise (so every tie goes to full attention)."""
    alpha = np.asarray(alpha, dtype=np.float64)
    a1, a2, a3 = alpha[..., 0], alpha[..., 1], alpha[..., 2]
    r = np.zeros(alpha.shape[:-1], dtype=np.uint8)
    r[(a2 > a1) & (a2 > a3)] = ROUTE_WINDOW
    r[(a3 > a1) & (a3 > a2)] = ROUTE_CORESET
    return r


def head_attention(route: int, Q, K, V, spec: LayerSpec, rows=None) -> np.ndarray:
    if route == ROUTE_FULL:
        return full_attention(Q, K, V, spec, rows)
    if route == ROUTE_WINDOW:
        return window_attention(Q, K, V, spec, rows)
    if route == ROUTE_CORESET:
        return coreset_attention(Q, K, V, spec, rows)
    raise ValueError(f"route {route}")


def routed_attention_layer(Q, K, V, routes: Sequence[int], spec: LayerSpec, rows=None) -> np.ndarray:
    """Eq. 4 applied per head.  Q, K, V: [heads, N, d] (anything np.asarray
    takes; widened to fp64 one head at a time).  rows: None (all), one index
    array for every head, or a dict head -> index array.  Returns
    [heads, n_rows, d] fp64 (a list of arrays if row counts differ)."""
    outs = []
    for h, route in enumerate(routes):
        r = rows.get(h) if isinstance(rows, dict) else rows
        outs.append(head_attention(int(route), np.asarray(Q[h], dtype=np.float64),
                                   np.asarray(K[h], dtype=np.float64),
                                   np.asarray(V[h], dtype=np.float64), spec, r))
    if len({o.shape for o in outs}) == 1:
        return np.stack(outs)
    return outs


def soft_mixture_layer(Q, K, V, alpha, spec: LayerSpec, rows=None) -> np.ndarray:
    """Eq. 5: every head runs all three branches, blended by its gates.
    alpha: [heads, 3]."""
    alpha = np.asarray(alpha, dtype=np.float64)
    outs = []
    for h in range(len(alpha)):
        q, k, v = (np.asarray(x[h], dtype=np.float64) for x in (Q, K, V))
        outs.append(sum(alpha[h, r] * head_attention(r, q, k, v, spec, rows) for r in range(3)))
    return np.stack(outs)
