// Host side of libvorta: plan construction, integer index tables, route bookkeeping.
// Nothing in this file touches the GPU.
#include <algorithm>
#include <array>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <new>

#include "vorta_internal.h"

namespace vorta {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = 0; }

void (*g_release_device_tables)(vorta_plan* p) = nullptr;

int split_routes(const vorta_plan* p, const uint8_t* routes, RouteLists* out) {
  if (!p || !routes || !out) return fail(VORTA_EINVAL, "null plan or routes");
  *out = RouteLists();
  for (int h = 0; h < p->d.heads; ++h) {
    int r = routes[h];
    if (r > 2) return fail(VORTA_EROUTE, "routes[%d] = %d, expected 0, 1 or 2", h, r);
    out->heads[r][out->count[r]++] = h;
  }
  return VORTA_OK;
}

UserTensor user_tensor(const vorta_plan* p, const void* base) {
  UserTensor t;
  t.base = base;
  const int64_t d = p->d.head_dim;
  if (p->d.layout == VORTA_LAYOUT_NHD) {
    t.head_stride = d;
    t.row_stride = (int64_t)p->d.heads * d;
  } else {
    t.head_stride = p->N * d;
    t.row_stride = d;
  }
  return t;
}

}  // namespace vorta

using namespace vorta;

extern "C" {

const char* vorta_strerror(int code) {
  switch (code) {
    case VORTA_OK: return "ok";
    case VORTA_EINVAL: return "invalid argument";
    case VORTA_ESHAPE: return "unsupported shape";
    case VORTA_EDTYPE: return "unsupported dtype";
    case VORTA_EWORKSPACE: return "workspace too small";
    case VORTA_EROUTE: return "invalid route code";
    case VORTA_EHIP: return "HIP runtime error";
    case VORTA_EALIGN: return "pointer not 16-byte aligned";
    default: return "unknown error";
  }
}

const char* vorta_last_error(void) { return g_err; }

// Window centre of Algorithm 1's get_window_center_id: "clamp" keeps the window inside the
// tile grid, "identity" leaves the query tile as the centre, "block" gives every query tile of a
// block of w tiles the block's middle tile (section 3.2's tau(i) per axis; the centre of a
// partial last block may lie past the grid).
static int window_centre(int q, int n, int w, int mode) {
  if (mode == VORTA_CENTER_IDENTITY) return q;
  if (mode == VORTA_CENTER_BLOCK) return q - q % w + w / 2;
  const int half = w / 2;
  const int lo = half, hi = std::max(n - 1 - half, half);
  return std::min(std::max(q, lo), hi);
}

int vorta_plan_create(const vorta_layer_desc* desc, vorta_plan** out) {
  clear_error();
  if (!desc || !out) return fail(VORTA_EINVAL, "null desc or out");
  *out = nullptr;
  vorta_layer_desc d = *desc;
  if (d.F < 1 || d.H < 1 || d.W < 1 || d.n_text < 0)
    return fail(VORTA_ESHAPE, "grid %dx%dx%d / n_text %d must be positive", d.F, d.H, d.W, d.n_text);
  {
    // axis by axis, so that no product leaves the range of int64
    const int64_t cap = (int64_t)1 << 30;
    int64_t tokens = d.F;
    for (int64_t axis : {(int64_t)d.H, (int64_t)d.W}) {
      if (tokens > cap || axis > cap) return fail(VORTA_ESHAPE, "more than 2^30 tokens");
      tokens *= axis;
    }
    if (tokens + d.n_text > cap) return fail(VORTA_ESHAPE, "more than 2^30 tokens");
  }
  if (d.heads < 1 || d.heads > VORTA_MAX_HEADS)
    return fail(VORTA_ESHAPE, "heads = %d, supported 1..%d", d.heads, VORTA_MAX_HEADS);
  if (d.dtype != VORTA_F32 && d.dtype != VORTA_BF16) return fail(VORTA_EDTYPE, "dtype %d", d.dtype);
  if (d.dtype == VORTA_BF16 && d.head_dim != 128)
    return fail(VORTA_ESHAPE, "bf16 supports head_dim 128, got %d", d.head_dim);
  if (d.dtype == VORTA_F32 && d.head_dim != 64 && d.head_dim != 128)
    return fail(VORTA_ESHAPE, "fp32 supports head_dim 64 or 128, got %d", d.head_dim);
  if (d.layout != VORTA_LAYOUT_NHD && d.layout != VORTA_LAYOUT_HND)
    return fail(VORTA_EINVAL, "layout %d", d.layout);
  if (d.center_mode != VORTA_CENTER_CLAMP && d.center_mode != VORTA_CENTER_IDENTITY &&
      d.center_mode != VORTA_CENTER_BLOCK)
    return fail(VORTA_EINVAL, "center_mode %d", d.center_mode);
  const int grid[3] = {d.F, d.H, d.W};
  int64_t bucket_tokens = 1, tile_tokens = 1;
  for (int a = 0; a < 3; ++a) {
    if (d.tile[a] < 1) return fail(VORTA_ESHAPE, "tile[%d] = %d < 1", a, d.tile[a]);
    if (d.window[a] < 1) return fail(VORTA_ESHAPE, "window[%d] = %d < 1", a, d.window[a]);
    if (d.bucket[a] < 1) return fail(VORTA_ESHAPE, "bucket[%d] = %d < 1", a, d.bucket[a]);
    // A tile or bucket larger than the axis is one clipped tile / bucket; a window of 2 n + 1
    // tiles or more sees the whole axis under every centre rule.  From here on the plan works
    // with the clipped values, so no product or sum below can leave the range of the grid.
    d.tile[a] = std::min(d.tile[a], grid[a]);
    d.bucket[a] = std::min(d.bucket[a], grid[a]);
    const int n_axis = (grid[a] + d.tile[a] - 1) / d.tile[a];
    d.window[a] = (int)std::min<int64_t>(d.window[a], 2 * (int64_t)n_axis + 1);
    bucket_tokens *= d.bucket[a];
    tile_tokens *= d.tile[a];
  }
  if (bucket_tokens > 64) return fail(VORTA_ESHAPE, "bucket holds %lld tokens, at most 64", (long long)bucket_tokens);
  if (d.keep_num < 1 || d.keep_den < d.keep_num)
    return fail(VORTA_ESHAPE, "core-set ratio %d/%d outside (0, 1]", d.keep_num, d.keep_den);
  int64_t rope_sum = 0;
  for (int a = 0; a < 3; ++a) {
    if (d.rope_dims[a] < 0 || d.rope_dims[a] % 2 || d.rope_dims[a] > d.head_dim)
      return fail(VORTA_ESHAPE, "rope_dims[%d] = %d: an even channel count in 0..head_dim expected", a, d.rope_dims[a]);
    rope_sum += d.rope_dims[a];
  }
  if (rope_sum > d.head_dim)
    return fail(VORTA_ESHAPE, "rope_dims add up to %lld channels, the head has %d", (long long)rope_sum, d.head_dim);
  if (!(d.rope_theta > 0.f)) d.rope_theta = 10000.f;

  {
    // the kernels address rows of a head with 32-bit element offsets (row index times row stride)
    const int64_t n_tokens = (int64_t)d.F * d.H * d.W + d.n_text;
    const int64_t row_stride = d.layout == VORTA_LAYOUT_NHD ? (int64_t)d.heads * d.head_dim : d.head_dim;
    if (n_tokens * row_stride > 0x7fffffffLL)
      return fail(VORTA_ESHAPE, "%lld tokens x row stride %lld elements exceed 2^31 elements per tensor",
                  (long long)n_tokens, (long long)row_stride);
  }
  vorta_plan* p = new (std::nothrow) vorta_plan();
  if (!p) return fail(VORTA_EINVAL, "out of host memory");
  p->d = d;
  p->L = (int64_t)d.F * d.H * d.W;
  p->N = p->L + d.n_text;
  p->elem_bytes = d.dtype == VORTA_BF16 ? 2 : 4;
  p->scale = d.softmax_scale > 0.f ? d.softmax_scale : (float)(1.0 / std::sqrt((double)d.head_dim));
  p->tile_tokens = (int)tile_tokens;   // <= L <= 2^30: every tile extent is clipped to its axis
  for (int a = 0; a < 3; ++a) {
    p->nt[a] = (grid[a] + d.tile[a] - 1) / d.tile[a];   // the last tile of an axis is clipped to the grid
    p->nb[a] = (grid[a] + d.bucket[a] - 1) / d.bucket[a];
  }
  p->n_tiles = p->nt[0] * p->nt[1] * p->nt[2];
  p->n_buckets = p->nb[0] * p->nb[1] * p->nb[2];

  // Tile order: tiles in raster order of their ids, the tokens of a tile in raster order of
  // their local coordinates; tile_row0 = first row of each tile.
  p->tile_row0.resize((size_t)p->n_tiles + 1);
  {
    int64_t row = 0;
    int t = 0;
    for (int tf = 0; tf < p->nt[0]; ++tf)
      for (int th = 0; th < p->nt[1]; ++th)
        for (int tw = 0; tw < p->nt[2]; ++tw) {
          p->tile_row0[t++] = (int32_t)row;
          row += (int64_t)std::min(d.tile[0], d.F - tf * d.tile[0]) * std::min(d.tile[1], d.H - th * d.tile[1]) *
                 std::min(d.tile[2], d.W - tw * d.tile[2]);
        }
    p->tile_row0[t] = (int32_t)row;   // = L
  }

  // Algorithm 1: key-tile box of every query tile.
  p->boxes.resize((size_t)p->n_tiles * 6);
  std::vector<std::vector<int32_t>> run_lists(p->n_tiles);
  p->window_key_tiles = 0;
  for (int qf = 0; qf < p->nt[0]; ++qf)
    for (int qh = 0; qh < p->nt[1]; ++qh)
      for (int qw = 0; qw < p->nt[2]; ++qw) {
        const int q[3] = {qf, qh, qw};
        const int tile = (qf * p->nt[1] + qh) * p->nt[2] + qw;
        int lo[3], hi[3];
        for (int a = 0; a < 3; ++a) {
          const int c = window_centre(q[a], p->nt[a], d.window[a], d.center_mode);
          const int half = d.window[a] / 2;   // abs(c - k) is an integer: <= w/2  <=>  <= floor(w/2)
          lo[a] = std::max(c - half, 0);
          hi[a] = std::min(c + half, p->nt[a] - 1);
          p->boxes[(size_t)tile * 6 + 2 * a] = lo[a];
          p->boxes[(size_t)tile * 6 + 2 * a + 1] = hi[a];
        }
        p->window_key_tiles = std::max(p->window_key_tiles,
                                       (hi[0] - lo[0] + 1) * (hi[1] - lo[1] + 1) * (hi[2] - lo[2] + 1));
        // Rows of a tile-ordered buffer: tiles along W are adjacent, so each (kf, kh) pair of
        // the box is one run; adjacent runs are merged.
        std::vector<int32_t>& rl = run_lists[tile];
        auto push = [&rl](int64_t start, int64_t len) {
          if (!rl.empty() && (int64_t)rl[rl.size() - 2] + rl[rl.size() - 1] == start) {
            rl[rl.size() - 1] += (int32_t)len;
          } else {
            rl.push_back((int32_t)start);
            rl.push_back((int32_t)len);
          }
        };
        for (int kf = lo[0]; kf <= hi[0]; ++kf)
          for (int kh = lo[1]; kh <= hi[1]; ++kh) {
            const int row_of_tiles = (kf * p->nt[1] + kh) * p->nt[2];
            const int64_t first = p->tile_row0[row_of_tiles + lo[2]];
            push(first, p->tile_row0[row_of_tiles + hi[2] + 1] - first);
          }
        if (d.n_text > 0) push(p->L, d.n_text);
      }
  p->max_runs = 1;
  for (auto& rl : run_lists) p->max_runs = std::max(p->max_runs, (int)rl.size() / 2);
  p->runs.assign((size_t)p->n_tiles * p->max_runs * 2, 0);
  p->n_runs.resize(p->n_tiles);
  for (int t = 0; t < p->n_tiles; ++t) {
    p->n_runs[t] = (int32_t)run_lists[t].size() / 2;
    std::copy(run_lists[t].begin(), run_lists[t].end(), p->runs.begin() + (size_t)t * p->max_runs * 2);
  }

  // Window work items.  Query tiles whose run lists are identical see the same keys (under the
  // clamped centre rule the border tile and its inner neighbour on every axis, under the block
  // rule all tiles of a block): they are computed together, greedily up to three tiles and 256
  // rows per item, so that one pass over the key stream serves them all.
  if (p->tile_tokens <= 128) {
    std::map<std::vector<int32_t>, std::vector<int>> same_keys;
    for (int t = 0; t < p->n_tiles; ++t) same_keys[run_lists[t]].push_back(t);
    std::vector<std::array<int32_t, 4>> big, small;
    auto flush = [&](std::array<int32_t, 4>& item, int rows) {
      if (item[3] == 0) return;
      (rows > 128 ? big : small).push_back(item);
      item = {0, 0, 0, 0};
    };
    for (auto& group : same_keys) {
      std::array<int32_t, 4> item = {0, 0, 0, 0};
      int rows = 0;
      for (int t : group.second) {                       // ascending tile ids
        const int n = p->tile_row0[t + 1] - p->tile_row0[t];
        if (item[3] == 3 || rows + n > 256) {
          flush(item, rows);
          rows = 0;
        }
        item[item[3]++] = t;
        rows += n;
      }
      flush(item, rows);
    }
    auto by_first_tile = [](const std::array<int32_t, 4>& a, const std::array<int32_t, 4>& b) { return a[0] < b[0]; };
    std::sort(big.begin(), big.end(), by_first_tile);    // neighbours in the list are neighbours on the grid
    std::sort(small.begin(), small.end(), by_first_tile);
    p->n_win_big = (int)big.size();
    p->n_win_small = (int)small.size();
    for (auto* list : {&big, &small})
      for (auto& item : *list) p->win_items.insert(p->win_items.end(), item.begin(), item.end());
  }

  // BCS slot layout: a (border-clipped) bucket of B' tokens keeps B' - k of them,
  // k = min(B' - 1, floor(B' (den - num) / den)).
  p->slot_base.resize((size_t)p->n_buckets + 1);
  int64_t slot = 0;
  int b = 0;
  for (int f0 = 0; f0 < d.F; f0 += d.bucket[0])
    for (int h0 = 0; h0 < d.H; h0 += d.bucket[1])
      for (int w0 = 0; w0 < d.W; w0 += d.bucket[2]) {
        const int B = std::min(d.bucket[0], d.F - f0) * std::min(d.bucket[1], d.H - h0) *
                      std::min(d.bucket[2], d.W - w0);
        const int k = std::min(B - 1, (int)(((int64_t)B * (d.keep_den - d.keep_num)) / d.keep_den));
        p->slot_base[b++] = (int32_t)slot;
        slot += B - k;
      }
  p->slot_base[b] = (int32_t)slot;
  p->Lc = slot;

  // rotary embedding table: (cos, sin) of position * theta^(-2 i / span), angles in double
  p->rope = rope_sum > 0;
  if (p->rope) {
    for (int a = 0; a < 3; ++a) {
      const int span = d.rope_dims[a];
      for (int pos = 0; pos < grid[a]; ++pos)
        for (int i = 0; i < span / 2; ++i) {
          const double angle = (double)pos * std::pow((double)d.rope_theta, -2.0 * i / span);
          p->rope_cs.push_back((float)std::cos(angle));
          p->rope_cs.push_back((float)std::sin(angle));
        }
    }
  }
  *out = p;
  return VORTA_OK;
}

int vorta_plan_destroy(vorta_plan* p) {
  clear_error();
  if (!p) return VORTA_OK;
  if (p->on_device && g_release_device_tables) g_release_device_tables(p);
  delete p;
  return VORTA_OK;
}

int vorta_plan_info_get(const vorta_plan* p, vorta_plan_info* out) {
  clear_error();
  if (!p || !out) return fail(VORTA_EINVAL, "null plan or out");
  out->n_video = p->L;
  out->n_tokens = p->N;
  for (int a = 0; a < 3; ++a) out->tiles[a] = p->nt[a];
  out->n_tiles = p->n_tiles;
  out->tile_tokens = p->tile_tokens;
  out->window_key_tiles = p->window_key_tiles;
  out->max_runs = p->max_runs;
  out->n_buckets = p->n_buckets;
  out->n_core = p->Lc;
  out->n_core_tokens = p->Lc + p->d.n_text;
  out->elem_bytes = p->elem_bytes;
  return VORTA_OK;
}

int vorta_tile_permutation(const vorta_plan* p, int32_t* perm) {
  clear_error();
  if (!p || !perm) return fail(VORTA_EINVAL, "null plan or perm");
  const vorta_layer_desc& d = p->d;
  int64_t i = 0;
  for (int f = 0; f < d.F; ++f)
    for (int h = 0; h < d.H; ++h)
      for (int w = 0; w < d.W; ++w, ++i) {
        const int tf = f / d.tile[0], th = h / d.tile[1], tw = w / d.tile[2];
        const int tile = (tf * p->nt[1] + th) * p->nt[2] + tw;
        const int ext_h = std::min(d.tile[1], d.H - th * d.tile[1]);   // extents of this (possibly clipped) tile
        const int ext_w = std::min(d.tile[2], d.W - tw * d.tile[2]);
        const int local = ((f % d.tile[0]) * ext_h + h % d.tile[1]) * ext_w + w % d.tile[2];
        perm[i] = p->tile_row0[tile] + local;
      }
  return VORTA_OK;
}

int vorta_tile_row0(const vorta_plan* p, int32_t* tile_row0) {
  clear_error();
  if (!p || !tile_row0) return fail(VORTA_EINVAL, "null plan or tile_row0");
  std::copy(p->tile_row0.begin(), p->tile_row0.end(), tile_row0);
  return VORTA_OK;
}

int vorta_window_boxes(const vorta_plan* p, int32_t* boxes) {
  clear_error();
  if (!p || !boxes) return fail(VORTA_EINVAL, "null plan or boxes");
  std::copy(p->boxes.begin(), p->boxes.end(), boxes);
  return VORTA_OK;
}

int vorta_window_runs(const vorta_plan* p, int32_t* runs, int32_t* n_runs) {
  clear_error();
  if (!p || !runs || !n_runs) return fail(VORTA_EINVAL, "null argument");
  std::copy(p->runs.begin(), p->runs.end(), runs);
  std::copy(p->n_runs.begin(), p->n_runs.end(), n_runs);
  return VORTA_OK;
}

int vorta_window_items(const vorta_plan* p, int32_t* items, int32_t counts[2]) {
  clear_error();
  if (!p || !counts) return fail(VORTA_EINVAL, "null argument");
  counts[0] = p->n_win_big;
  counts[1] = p->n_win_small;
  if (items) std::copy(p->win_items.begin(), p->win_items.end(), items);
  return VORTA_OK;
}

int vorta_bcs_slot_bases(const vorta_plan* p, int32_t* slot_base) {
  clear_error();
  if (!p || !slot_base) return fail(VORTA_EINVAL, "null argument");
  std::copy(p->slot_base.begin(), p->slot_base.end(), slot_base);
  return VORTA_OK;
}

int vorta_route_partition(const vorta_plan* p, const uint8_t* routes_host, int32_t* heads_by_route,
                          int32_t counts[3]) {
  clear_error();
  if (!heads_by_route || !counts) return fail(VORTA_EINVAL, "null output");
  RouteLists rl;
  if (int rc = split_routes(p, routes_host, &rl)) return rc;
  int n = 0;
  for (int r = 0; r < 3; ++r) {
    counts[r] = rl.count[r];
    for (int i = 0; i < rl.count[r]; ++i) heads_by_route[n++] = rl.heads[r][i];
  }
  return VORTA_OK;
}

int vorta_router_gates(const float* t_emb, const float* w_r, int32_t d_t, int32_t heads, float* alpha_out) {
  clear_error();
  if (!t_emb || !w_r || !alpha_out || heads < 0) return fail(VORTA_EINVAL, "null argument");
  if (d_t < 1) return fail(VORTA_EINVAL, "d_t = %d: the timestep embedding is empty", d_t);
  for (int h = 0; h < heads; ++h) {
    const float* w = w_r + (size_t)h * d_t * 3;
    double z[3] = {0.0, 0.0, 0.0};
    for (int i = 0; i < d_t; ++i)
      for (int k = 0; k < 3; ++k) z[k] += (double)t_emb[i] * (double)w[3 * i + k];
    const double m = std::max(z[0], std::max(z[1], z[2]));
    double e[3], sum = 0.0;
    for (int k = 0; k < 3; ++k) { e[k] = std::exp(z[k] - m); sum += e[k]; }
    for (int k = 0; k < 3; ++k) alpha_out[3 * h + k] = (float)(e[k] / sum);
  }
  return VORTA_OK;
}

int vorta_route_select(const float* alpha, int32_t heads, uint8_t* routes) {
  clear_error();
  if (!alpha || !routes || heads < 0) return fail(VORTA_EINVAL, "null argument");
  for (int h = 0; h < heads; ++h) {
    const float a1 = alpha[3 * h], a2 = alpha[3 * h + 1], a3 = alpha[3 * h + 2];
    uint8_t r = VORTA_ROUTE_FULL;
    if (a2 > a1 && a2 > a3) r = VORTA_ROUTE_WINDOW;
    else if (a3 > a1 && a3 > a2) r = VORTA_ROUTE_CORESET;
    routes[h] = r;
  }
  return VORTA_OK;
}

// Workspace: q_t,k_t,v_t,o_t,q_c,k_c,v_c,o_c,keep_idx,assign,q_r,k_r, each 256-byte aligned.
static void workspace_sizes(const vorta_plan* p, const RouteLists& rl, size_t sizes[12]) {
  const size_t row = (size_t)p->d.head_dim * p->elem_bytes;
  // tile-ordered copies: only the fp32 layer call makes them (bf16 gathers rows in the window kernel)
  const size_t tiled = p->d.dtype == VORTA_BF16 ? 0 : (size_t)rl.count[1] * p->N * row;
  const size_t core = (size_t)rl.count[2] * (p->Lc + p->d.n_text) * row;
  for (int i = 0; i < 4; ++i) sizes[i] = tiled;
  for (int i = 4; i < 8; ++i) sizes[i] = core;
  sizes[8] = (size_t)rl.count[2] * p->Lc * sizeof(int32_t);
  sizes[9] = (size_t)rl.count[2] * p->L * sizeof(int32_t);
  // rotated copies of Q and K for the heads on routes 0 and 1: whole tensors in the caller's
  // layout (rows of the other heads stay unwritten), so that the attention kernels address
  // them with the strides they use for V and the output
  sizes[10] = sizes[11] = p->rope && rl.count[0] + rl.count[1] ? (size_t)p->d.heads * p->N * row : 0;
}

int vorta_workspace_layout(const vorta_plan* p, const uint8_t* routes_host, size_t offsets[12]) {
  clear_error();
  if (!offsets) return fail(VORTA_EINVAL, "null offsets");
  RouteLists rl;
  if (int rc = split_routes(p, routes_host, &rl)) return rc;
  size_t sizes[12], off = 0;
  workspace_sizes(p, rl, sizes);
  for (int i = 0; i < 12; ++i) {
    offsets[i] = off;
    off += (sizes[i] + 255) & ~(size_t)255;
  }
  return VORTA_OK;
}

int vorta_workspace_bytes(const vorta_plan* p, const uint8_t* routes_host, size_t* bytes) {
  clear_error();
  if (!bytes) return fail(VORTA_EINVAL, "null bytes");
  RouteLists rl;
  if (int rc = split_routes(p, routes_host, &rl)) return rc;
  size_t sizes[12], off = 0;
  workspace_sizes(p, rl, sizes);
  for (int i = 0; i < 12; ++i) off += (sizes[i] + 255) & ~(size_t)255;
  *bytes = off + 256;   // never zero, so callers can always allocate it
  return VORTA_OK;
}

int vorta_soft_mixture_workspace_bytes(const vorta_plan* p, size_t* bytes) {
  clear_error();
  if (!p || !bytes) return fail(VORTA_EINVAL, "null argument");
  uint8_t routes[VORTA_MAX_HEADS];
  if (p->d.dtype == VORTA_BF16) {
    // fused form: the core-set buffers and index of every head (and, with a rotary embedding,
    // the rotated copies of Q and K)
    std::memset(routes, VORTA_ROUTE_CORESET, sizeof(routes));
    if (int rc = vorta_workspace_bytes(p, routes, bytes)) return rc;
    if (p->rope) *bytes += 2 * (((size_t)p->d.heads * p->N * p->d.head_dim * p->elem_bytes + 255) & ~(size_t)255);
    return VORTA_OK;
  }
  // fp32: the largest single-route workspace + one user-layout output per branch
  size_t most = 0;
  for (int r = 0; r < 3; ++r) {
    std::memset(routes, r, sizeof(routes));
    size_t b = 0;
    if (int rc = vorta_workspace_bytes(p, routes, &b)) return rc;
    most = std::max(most, b);
  }
  const size_t out_bytes = ((size_t)p->d.heads * p->N * p->d.head_dim * p->elem_bytes + 255) & ~(size_t)255;
  *bytes = most + 3 * out_bytes;
  return VORTA_OK;
}

}  // extern "C"
