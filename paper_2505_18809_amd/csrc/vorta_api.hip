// Device entry points of libvorta: argument checks, workspace carving, launch sequencing.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "vorta_attn_common.h"

namespace vorta {

static int check_ptr(const void* p, const char* name) {
  if (!p) return fail(VORTA_EINVAL, "%s is null", name);
  if ((uintptr_t)p & 15) return fail(VORTA_EALIGN, "%s = %p is not 16-byte aligned", name, p);
  return VORTA_OK;
}

#define VORTA_TRY(expr)        \
  do {                         \
    if (int rc_ = (expr)) return rc_; \
  } while (0)

// Scratch of the entry point that allocates nothing: a fixed array in the library's own device
// image, one copy per GPU at an address of its own.  In host code the array's name is only a
// stand-in for the symbol; the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[VORTA_STATIC_SCRATCH_BYTES];

static int static_scratch(void** out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void* ptr[MAX_DEVICES] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(VORTA_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(VORTA_EINVAL, "device %d: at most %d devices", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* found = nullptr;
    e = hipGetSymbolAddress(&found, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !found)
      return fail(VORTA_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    ptr[dev] = found;
  }
  *out = ptr[dev];
  return VORTA_OK;
}

static int begin(vorta_plan* p, const uint8_t* routes, RouteLists* rl) {
  clear_error();
  VORTA_TRY(split_routes(p, routes, rl));
  return ensure_device_tables(p);
}

int fill_attn_args(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, int BM, int win_part, AttnArgs* a,
                   int win_list) {
  std::memset(a, 0, sizeof(*a));
  const UserTensor ut = user_tensor(p, io->q);
  a->q0 = io->q; a->k0 = io->k; a->v0 = io->v; a->o0 = io->out;
  a->head_stride0 = ut.head_stride;
  a->row_stride0 = ut.row_stride;
  a->qc = io->q_c; a->kc = io->k_c; a->vc = io->v_c; a->oc = io->o_c;
  a->qt = io->q_t; a->kt = io->k_t; a->vt = io->v_t; a->ot = io->o_t;
  a->tok_of = p->d_tok_of;
  a->tile_row0 = p->d_tile_row0;
  a->win_gather = io->q_t == nullptr;
  a->runs = p->d_runs;
  a->n_runs = p->d_n_runs;
  a->max_runs = p->max_runs;
  a->N = (int)p->N;
  a->Nc = (int)(p->Lc + p->d.n_text);
  a->L = (int)p->L;
  a->n_text = p->d.n_text;
  a->n_tiles = p->n_tiles;
  a->tile_tokens = p->tile_tokens;
  a->qb_dense = (a->N + BM - 1) / BM;
  a->qb_core = (a->Nc + BM - 1) / BM;
  a->qb_tile = (a->tile_tokens + BM - 1) / BM;
  a->qb_text = (a->n_text + BM - 1) / BM;
  const long end_text = win_part & WIN_TEXT ? (long)rl.count[1] * a->qb_text : 0;
  const long end_dense = end_text + (long)rl.count[0] * a->qb_dense;
  const long end_core = end_dense + (long)rl.count[2] * a->qb_core;
  long tile_items = (long)a->n_tiles * a->qb_tile;        // per window head
  if (win_list >= 0) {
    a->win_items = p->d_win_items;
    a->win_first = win_list == 0 ? 0 : p->n_win_big;
    a->win_count = win_list == 0 ? p->n_win_big : p->n_win_small;
    tile_items = a->win_count;
  }
  const long end_tile = end_core + (win_part & WIN_TILES ? (long)rl.count[1] * tile_items : 0);
  if (end_tile > 0x7fffffffL) return fail(VORTA_ESHAPE, "%ld work items exceed the grid limit", end_tile);
  a->end_text = (int)end_text;
  a->end_dense = (int)end_dense;
  a->end_core = (int)end_core;
  a->end_tile = (int)end_tile;
  a->split_from = 0x7fffffff;
  a->scale = p->scale;
  for (int i = 0; i < rl.count[0]; ++i) a->dense_heads[i] = (uint8_t)rl.heads[0][i];
  for (int i = 0; i < rl.count[1]; ++i) a->win_heads[i] = (uint8_t)rl.heads[1][i];
  return VORTA_OK;
}

static int attention(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream) {
  if (!io) return fail(VORTA_EINVAL, "io is null");
  const bool gather = rl.count[1] && !io->q_t && !io->k_t && !io->v_t && !io->o_t;   // window heads read q, k, v directly
  if (gather && p->d.dtype != VORTA_BF16)
    return fail(VORTA_EINVAL, "the fp32 path needs the tile-ordered copies io.q_t, k_t, v_t, o_t");
  if (rl.count[0] || gather) {
    VORTA_TRY(check_ptr(io->q, "io.q")); VORTA_TRY(check_ptr(io->k, "io.k"));
    VORTA_TRY(check_ptr(io->v, "io.v")); VORTA_TRY(check_ptr(io->out, "io.out"));
  }
  if (rl.count[1] && !gather) {
    VORTA_TRY(check_ptr(io->q_t, "io.q_t")); VORTA_TRY(check_ptr(io->k_t, "io.k_t"));
    VORTA_TRY(check_ptr(io->v_t, "io.v_t")); VORTA_TRY(check_ptr(io->o_t, "io.o_t"));
  }
  if (rl.count[2]) {
    VORTA_TRY(check_ptr(io->q_c, "io.q_c")); VORTA_TRY(check_ptr(io->k_c, "io.k_c"));
    VORTA_TRY(check_ptr(io->v_c, "io.v_c")); VORTA_TRY(check_ptr(io->o_c, "io.o_c"));
  }
  return p->d.dtype == VORTA_BF16 ? launch_attention_bf16(p, rl, io, stream)
                                  : launch_attention_f32(p, rl, io, stream);
}

struct Carved {
  char* buf[12];
};

static int carve(const vorta_plan* p, const uint8_t* routes, void* workspace, size_t bytes, Carved* c) {
  size_t need = 0, off[12];
  VORTA_TRY(vorta_workspace_bytes(p, routes, &need));
  if (bytes < need) return fail(VORTA_EWORKSPACE, "workspace has %zu bytes, need %zu", bytes, need);
  VORTA_TRY(check_ptr(workspace, "workspace"));
  VORTA_TRY(vorta_workspace_layout(p, routes, off));
  for (int i = 0; i < 12; ++i) c->buf[i] = (char*)workspace + off[i];
  return VORTA_OK;
}

// Route 2, first half: core-set index on K as given (before any rotation), then Q, K, V pooled;
// the pooled rows of Q and K are rotated at their slot owner's position.  One fused pass where
// the bucket is small enough, else the index pass and three pool passes.
static int select_and_pool(vorta_plan* p, const RouteLists& rl, const void* q, const void* k, const void* v,
                           int32_t* keep_idx, int32_t* assign, const Carved& c, void* stream) {
  if (bcs_fused_applies(p))
    return launch_bcs_select_pool(p, rl, q, k, v, keep_idx, assign, c.buf[4], c.buf[5], c.buf[6], stream);
  VORTA_TRY(launch_bcs_index(p, rl, user_tensor(p, k), keep_idx, assign, stream));
  VORTA_TRY(launch_bcs_pool(p, rl, q, keep_idx, assign, true, c.buf[4], stream));
  VORTA_TRY(launch_bcs_pool(p, rl, k, keep_idx, assign, true, c.buf[5], stream));
  return launch_bcs_pool(p, rl, v, keep_idx, assign, false, c.buf[6], stream);
}

static int layer(vorta_plan* p, const RouteLists& rl, const void* q, const void* k, const void* v,
                 const uint8_t* routes, void* out, const Carved& c, void* stream) {
  int32_t* keep_idx = (int32_t*)c.buf[8];
  int32_t* assign = (int32_t*)c.buf[9];
  // route 1: with bf16 the window kernel gathers token rows through the tile permutation and
  // scatters its output rows the same way, so the reorder passes and the tile-ordered copies
  // are only used by the fp32 path
  const bool gather = p->d.dtype == VORTA_BF16;
  // routes 0 and 1 with a rotary embedding: attention reads rotated copies of Q and K
  const void *q_att = q, *k_att = k;
  if (p->rope && rl.count[0] + rl.count[1] > 0) {
    VORTA_TRY(launch_rope_rows(p, rl, q, c.buf[10], stream));
    VORTA_TRY(launch_rope_rows(p, rl, k, c.buf[11], stream));
    q_att = c.buf[10];
    k_att = c.buf[11];
  }
  if (!gather) {
    VORTA_TRY(launch_reorder(p, rl, q_att, c.buf[0], true, stream));
    VORTA_TRY(launch_reorder(p, rl, k_att, c.buf[1], true, stream));
    VORTA_TRY(launch_reorder(p, rl, v, c.buf[2], true, stream));
  }
  VORTA_TRY(select_and_pool(p, rl, q, k, v, keep_idx, assign, c, stream));
  vorta_attn_io io;
  io.q = q_att; io.k = k_att; io.v = v; io.out = out;
  io.q_t = io.k_t = io.v_t = nullptr;
  io.o_t = nullptr;
  if (!gather) { io.q_t = c.buf[0]; io.k_t = c.buf[1]; io.v_t = c.buf[2]; io.o_t = c.buf[3]; }
  io.q_c = c.buf[4]; io.k_c = c.buf[5]; io.v_c = c.buf[6]; io.o_c = c.buf[7];
  VORTA_TRY(attention(p, rl, &io, stream));
  if (!gather) VORTA_TRY(launch_reorder(p, rl, out, c.buf[3], false, stream));
  VORTA_TRY(launch_unpool(p, rl, c.buf[7], assign, out, stream));
  (void)routes;
  return VORTA_OK;
}

}  // namespace vorta

using namespace vorta;

extern "C" {

int vorta_reorder_to_tiles(vorta_plan* p, const void* src, const uint8_t* routes, void* dst, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  if (!rl.count[1]) return VORTA_OK;
  VORTA_TRY(check_ptr(src, "src"));
  VORTA_TRY(check_ptr(dst, "dst"));
  return launch_reorder(p, rl, src, dst, true, stream);
}

int vorta_reorder_from_tiles(vorta_plan* p, const void* src, const uint8_t* routes, void* dst, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  if (!rl.count[1]) return VORTA_OK;
  VORTA_TRY(check_ptr(src, "src"));
  VORTA_TRY(check_ptr(dst, "dst"));
  return launch_reorder(p, rl, dst, const_cast<void*>(src), false, stream);
}

int vorta_bcs_build_index(vorta_plan* p, const void* feat, int64_t feat_head_stride, const uint8_t* routes,
                          int32_t* keep_idx, int32_t* assign, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  if (feat_head_stride < VORTA_FEAT_USER_LAYOUT)
    return fail(VORTA_EINVAL, "feat_head_stride = %lld: VORTA_FEAT_USER_LAYOUT, 0 or a positive stride", (long long)feat_head_stride);
  if (feat_head_stride > 0 && (feat_head_stride < p->L * p->d.head_dim || feat_head_stride % (16 / p->elem_bytes)))
    return fail(VORTA_EINVAL, "feat_head_stride = %lld: heads overlap (a head holds %lld elements) or lose 16-byte alignment",
                (long long)feat_head_stride, (long long)(p->L * p->d.head_dim));
  if (!rl.count[2]) return VORTA_OK;
  VORTA_TRY(check_ptr(feat, "feat"));
  VORTA_TRY(check_ptr(keep_idx, "keep_idx"));
  VORTA_TRY(check_ptr(assign, "assign"));
  UserTensor ut = user_tensor(p, feat);
  if (feat_head_stride != VORTA_FEAT_USER_LAYOUT) {   // [heads or 1][rows][head_dim]
    ut.head_stride = feat_head_stride;
    ut.row_stride = p->d.head_dim;
  }
  return launch_bcs_index(p, rl, ut, keep_idx, assign, stream);
}

int vorta_bcs_select_pool(vorta_plan* p, const void* q, const void* k, const void* v, const uint8_t* routes,
                          int32_t* keep_idx, int32_t* assign, void* q_c, void* k_c, void* v_c, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  if (!rl.count[2]) return VORTA_OK;
  VORTA_TRY(check_ptr(q, "q")); VORTA_TRY(check_ptr(k, "k")); VORTA_TRY(check_ptr(v, "v"));
  VORTA_TRY(check_ptr(keep_idx, "keep_idx")); VORTA_TRY(check_ptr(assign, "assign"));
  VORTA_TRY(check_ptr(q_c, "q_c")); VORTA_TRY(check_ptr(k_c, "k_c")); VORTA_TRY(check_ptr(v_c, "v_c"));
  Carved c;
  std::memset(&c, 0, sizeof(c));
  c.buf[4] = (char*)q_c; c.buf[5] = (char*)k_c; c.buf[6] = (char*)v_c;
  return select_and_pool(p, rl, q, k, v, keep_idx, assign, c, stream);
}

int vorta_rope_apply(vorta_plan* p, const void* src, const uint8_t* routes, void* dst, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  if (!p->rope || rl.count[0] + rl.count[1] == 0) return VORTA_OK;
  VORTA_TRY(check_ptr(src, "src"));
  VORTA_TRY(check_ptr(dst, "dst"));
  return launch_rope_rows(p, rl, src, dst, stream);
}

int vorta_bcs_pool(vorta_plan* p, const void* src, const uint8_t* routes, const int32_t* keep_idx,
                   const int32_t* assign, int32_t rotate, void* dst, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  if (!rl.count[2]) return VORTA_OK;
  VORTA_TRY(check_ptr(src, "src"));
  VORTA_TRY(check_ptr(keep_idx, "keep_idx"));
  VORTA_TRY(check_ptr(assign, "assign"));
  VORTA_TRY(check_ptr(dst, "dst"));
  return launch_bcs_pool(p, rl, src, keep_idx, assign, rotate != 0, dst, stream);
}

int vorta_attention_routed(vorta_plan* p, const uint8_t* routes, const vorta_attn_io* io, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  return attention(p, rl, io, stream);
}

int vorta_scatter_back(vorta_plan* p, const uint8_t* routes, const void* o_t, const void* o_c,
                       const int32_t* assign, void* out, void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  if (rl.count[1] || rl.count[2]) VORTA_TRY(check_ptr(out, "out"));
  if (rl.count[1] && !o_t && p->d.dtype != VORTA_BF16)
    return fail(VORTA_EINVAL, "o_t is null: only the bf16 window kernel writes its rows to `out` itself");
  if (rl.count[1] && o_t) {      // o_t null: the window heads wrote their rows to `out` themselves
    VORTA_TRY(check_ptr(o_t, "o_t"));
    VORTA_TRY(launch_reorder(p, rl, out, const_cast<void*>(o_t), false, stream));
  }
  if (rl.count[2]) {
    VORTA_TRY(check_ptr(o_c, "o_c"));
    VORTA_TRY(check_ptr(assign, "assign"));
    VORTA_TRY(launch_unpool(p, rl, o_c, assign, out, stream));
  }
  return VORTA_OK;
}

int vorta_routed_attention_layer(vorta_plan* p, const void* q, const void* k, const void* v,
                                 const uint8_t* routes, void* out, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  RouteLists rl;
  VORTA_TRY(begin(p, routes, &rl));
  VORTA_TRY(check_ptr(q, "q")); VORTA_TRY(check_ptr(k, "k"));
  VORTA_TRY(check_ptr(v, "v")); VORTA_TRY(check_ptr(out, "out"));
  Carved c;
  VORTA_TRY(carve(p, routes, workspace, workspace_bytes, &c));
  return layer(p, rl, q, k, v, routes, out, c, stream);
}

int vorta_soft_mixture_layer(vorta_plan* p, const void* q, const void* k, const void* v,
                             const float* alpha_host, void* out, void* workspace, size_t workspace_bytes,
                             void* stream) {
  clear_error();
  if (!p || !alpha_host) return fail(VORTA_EINVAL, "null plan or alpha");
  VORTA_TRY(check_ptr(q, "q")); VORTA_TRY(check_ptr(k, "k"));
  VORTA_TRY(check_ptr(v, "v")); VORTA_TRY(check_ptr(out, "out"));
  size_t need = 0;
  VORTA_TRY(vorta_soft_mixture_workspace_bytes(p, &need));
  if (workspace_bytes < need) return fail(VORTA_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, need);
  VORTA_TRY(check_ptr(workspace, "workspace"));
  uint8_t routes[VORTA_MAX_HEADS];
  if (p->d.dtype == VORTA_BF16) {
    // Fused form: no branch is written out in full and there is no blend pass.
    //   1. core-set branch of every head -> o_c (pooled rows only)
    //   2. sliding-tile branch of every head -> the video rows of `out`, unscaled
    //   3. full-attention branch of every head; its epilogue reads the row `out` holds and the
    //      row of o_c the token is assigned to, and writes a1 full + a2 sliding + a3 core-set.
    // The three run in this order on the stream, so each finds its inputs complete.
    RouteLists rl;
    Carved c;
    std::memset(routes, VORTA_ROUTE_CORESET, sizeof(routes));
    VORTA_TRY(begin(p, routes, &rl));
    VORTA_TRY(carve(p, routes, workspace, workspace_bytes, &c));
    int32_t* keep_idx = (int32_t*)c.buf[8];
    int32_t* assign = (int32_t*)c.buf[9];
    VORTA_TRY(select_and_pool(p, rl, q, k, v, keep_idx, assign, c, stream));
    const void *q_att = q, *k_att = k;
    if (p->rope) {       // rotated copies for the other two branches, behind the core-set buffers
      size_t core_bytes = 0;
      VORTA_TRY(vorta_workspace_bytes(p, routes, &core_bytes));
      const size_t tensor_bytes = ((size_t)p->d.heads * p->N * p->d.head_dim * p->elem_bytes + 255) & ~(size_t)255;
      char* q_r = (char*)workspace + core_bytes;
      char* k_r = q_r + tensor_bytes;
      RouteLists all_full;
      std::memset(routes, VORTA_ROUTE_FULL, sizeof(routes));
      VORTA_TRY(split_routes(p, routes, &all_full));
      VORTA_TRY(launch_rope_rows(p, all_full, q, q_r, stream));
      VORTA_TRY(launch_rope_rows(p, all_full, k, k_r, stream));
      q_att = q_r;
      k_att = k_r;
    }
    vorta_attn_io io;
    std::memset(&io, 0, sizeof(io));
    io.q = q_att; io.k = k_att; io.v = v; io.out = out;
    io.q_c = c.buf[4]; io.k_c = c.buf[5]; io.v_c = c.buf[6]; io.o_c = c.buf[7];
    VORTA_TRY(launch_attention_bf16(p, rl, &io, stream));
    std::memset(routes, VORTA_ROUTE_WINDOW, sizeof(routes));
    VORTA_TRY(split_routes(p, routes, &rl));
    VORTA_TRY(launch_attention_bf16(p, rl, &io, stream, nullptr, false));
    std::memset(routes, VORTA_ROUTE_FULL, sizeof(routes));
    VORTA_TRY(split_routes(p, routes, &rl));
    MixArgs mix;
    std::memset(&mix, 0, sizeof(mix));
    mix.oc = c.buf[7];
    mix.assign = assign;
    mix.Lc = (int)p->Lc;
    for (int h = 0; h < p->d.heads; ++h)
      for (int r = 0; r < 3; ++r) mix.alpha[h][r] = alpha_host[3 * h + r];
    return launch_attention_bf16(p, rl, &io, stream, &mix);
  }
  // fp32 (the exact path): every branch into a buffer of its own, then one blend pass
  const size_t out_bytes = ((size_t)p->d.heads * p->N * p->d.head_dim * p->elem_bytes + 255) & ~(size_t)255;
  char* branch[3] = {(char*)workspace, (char*)workspace + out_bytes, (char*)workspace + 2 * out_bytes};
  char* inner = (char*)workspace + 3 * out_bytes;
  const size_t inner_bytes = workspace_bytes - 3 * out_bytes;
  for (int r = 0; r < 3; ++r) {
    std::memset(routes, r, sizeof(routes));
    RouteLists rl;
    VORTA_TRY(begin(p, routes, &rl));
    Carved c;
    VORTA_TRY(carve(p, routes, inner, inner_bytes, &c));
    VORTA_TRY(layer(p, rl, q, k, v, routes, branch[r], c, stream));
  }
  return launch_blend3(p, branch[0], branch[1], branch[2], alpha_host, out, stream);
}

int vorta_plan_upload(vorta_plan* p) {
  clear_error();
  if (!p) return fail(VORTA_EINVAL, "null plan");
  VORTA_TRY(ensure_device_tables(p));
  void* scratch_ptr = nullptr;
  return static_scratch(&scratch_ptr);     // also resolves the static scratch of this device
}

int vorta_router_device(const float* t_emb, const float* w_r, int32_t n_steps, int32_t d_t, int32_t heads,
                        float* alpha, uint8_t* routes, uint8_t* routes_host, void* stream) {
  clear_error();
  if (n_steps < 1 || d_t < 1 || heads < 1 || heads > VORTA_MAX_HEADS || n_steps > 65535)
    return fail(VORTA_EINVAL, "n_steps = %d (1..65535), d_t = %d (>= 1), heads = %d (1..%d)", n_steps, d_t, heads, VORTA_MAX_HEADS);
  if (!t_emb || !w_r || !alpha || !routes) return fail(VORTA_EINVAL, "null argument");
  if (((uintptr_t)t_emb | (uintptr_t)w_r | (uintptr_t)alpha) & 3) return fail(VORTA_EALIGN, "float arrays must be 4-byte aligned");
  VORTA_TRY(launch_router(t_emb, w_r, n_steps, d_t, heads, alpha, routes, stream));
  if (routes_host) {
    hipError_t e = hipMemcpyAsync(routes_host, routes, (size_t)n_steps * heads, hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e != hipSuccess) return fail(VORTA_EHIP, "copy of the routes to the host: %s", hipGetErrorString(e));
  }
  return VORTA_OK;
}

int vorta_routed_attention_layer_static(vorta_plan* p, const void* q, const void* k, const void* v,
                                        const uint8_t* routes, void* out, void* stream) {
  clear_error();
  RouteLists rl;
  VORTA_TRY(split_routes(p, routes, &rl));
  {
    std::lock_guard<std::mutex> lock(p->mu);
    if (!p->on_device)
      return fail(VORTA_EINVAL, "the plan's tables are not on the device: call vorta_plan_upload once first (this call allocates nothing)");
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(VORTA_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev != p->device) return fail(VORTA_EINVAL, "plan belongs to device %d, current device is %d", p->device, dev);
  }
  VORTA_TRY(check_ptr(q, "q")); VORTA_TRY(check_ptr(k, "k"));
  VORTA_TRY(check_ptr(v, "v")); VORTA_TRY(check_ptr(out, "out"));
  size_t need = 0;
  VORTA_TRY(vorta_workspace_bytes(p, routes, &need));
  if (need > VORTA_STATIC_SCRATCH_BYTES)
    return fail(VORTA_EWORKSPACE, "this layer needs %zu bytes of scratch, the static buffer holds %zu: use vorta_routed_attention_layer with a workspace",
                need, (size_t)VORTA_STATIC_SCRATCH_BYTES);
  void* scratch_ptr = nullptr;
  VORTA_TRY(static_scratch(&scratch_ptr));
  Carved c;
  VORTA_TRY(carve(p, routes, scratch_ptr, VORTA_STATIC_SCRATCH_BYTES, &c));
  return layer(p, rl, q, k, v, routes, out, c, stream);
}

}  // extern "C"
