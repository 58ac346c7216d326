/*
 * vorta.h -- C ABI of the routed attention layer of VORTA (arXiv 2505.18809)
 * for AMD MI355X (gfx950).
 *
 * One layer call computes, for every head h of a video diffusion transformer
 * attention layer, the branch its route selects (Eq. 4):
 *     route 0  full 3-D attention                         (Eq. 2)
 *     route 1  3-D sliding tile attention                 (Algorithm 1)
 *     route 2  core-set attention  unpool . attn . pool   (section 3.2, Fig. 3)
 *
 * Conventions that hold for every call
 *   - Tokens: the F x H x W latent grid flattened frame-major (F slowest) into
 *     L video tokens, followed by n_text text tokens; N = L + n_text.
 *   - Tensors are dense arrays of `dtype` elements in `layout`:
 *     VORTA_LAYOUT_NHD = [N][heads][head_dim], VORTA_LAYOUT_HND =
 *     [heads][N][head_dim].  "user layout" below means this.
 *   - routes_host is a HOST array uint8[heads] with codes 0/1/2 (the router is
 *     a scalar-sized host decision).  Heads of one route are numbered by
 *     ascending head id ("slot"); internal per-route buffers are indexed by slot.
 *   - Every other data pointer is DEVICE memory owned by the caller, 16-byte
 *     aligned, alive until the stream work has finished.  The library never
 *     frees or keeps caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Device
 *     calls only enqueue work; they do not synchronise.  Exception: the first
 *     device call on a plan uploads the plan's small index tables with a
 *     blocking hipMalloc + hipMemcpy (a few hundred KB, once per plan) on the
 *     device that is current then; the plan belongs to that device from then on
 *     (a device call with another device current returns VORTA_EINVAL).  Call
 *     vorta_plan_upload beforehand to have that done at a time of your choosing
 *     (needed before the first call under graph capture).
 *   - Return value: VORTA_OK or a negative error code; vorta_last_error() has
 *     a thread-local message.  Nothing is printed, thrown or aborted.  Invalid
 *     arguments are rejected before any kernel is launched.
 *   - There is no CPU fallback: device calls on a machine without a usable
 *     gfx950 device fail with VORTA_EHIP.
 */
#ifndef VORTA_H
#define VORTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  VORTA_OK = 0,
  VORTA_EINVAL = -1,      /* null pointer, bad enum value                                  */
  VORTA_ESHAPE = -2,      /* grid, tile, window or bucket < 1, head_dim unsupported, too many tokens */
  VORTA_EDTYPE = -3,
  VORTA_EWORKSPACE = -4,  /* workspace smaller than vorta_workspace_bytes                   */
  VORTA_EROUTE = -5,      /* a route code above 2                                          */
  VORTA_EHIP = -6,        /* a HIP runtime call failed; message holds hipGetErrorString    */
  VORTA_EALIGN = -7       /* a device pointer is not 16-byte aligned                       */
};

enum { VORTA_ROUTE_FULL = 0, VORTA_ROUTE_WINDOW = 1, VORTA_ROUTE_CORESET = 2 };
enum { VORTA_F32 = 0, VORTA_BF16 = 1 };
enum { VORTA_LAYOUT_NHD = 0, VORTA_LAYOUT_HND = 1 };
/* Readings of Algorithm 1's get_window_center_id (named there, not defined), per axis, for query
 * tile q of n tiles under a window of w tiles:
 *   CLAMP     min(max(q, w/2), max(n - 1 - w/2, w/2)): the window slides but stays inside the grid
 *   IDENTITY  q: the window is cut off at the border
 *   BLOCK     (q / w) w + w/2: the tile grid is cut into blocks of w tiles whose query tiles all
 *             share the block's middle tile (section 3.2's tau(i) taken per axis on tile ids)   */
enum { VORTA_CENTER_CLAMP = 0, VORTA_CENTER_IDENTITY = 1, VORTA_CENTER_BLOCK = 2 };

#define VORTA_MAX_HEADS 128

/* Layer description: plain data, copied by vorta_plan_create. */
typedef struct vorta_layer_desc {
  int32_t F, H, W;          /* latent grid                                                   */
  int32_t n_text;           /* text tokens after the video tokens (0 = none)                 */
  int32_t heads;            /* 1 .. VORTA_MAX_HEADS                                          */
  int32_t head_dim;         /* bf16: 128; fp32: 64 or 128                                    */
  int32_t dtype;            /* VORTA_F32 | VORTA_BF16 (inputs, outputs and internal buffers) */
  int32_t layout;           /* VORTA_LAYOUT_*                                                */
  int32_t tile[3];          /* tokens per tile (t_F, t_H, t_W) >= 1; where a tile does not divide
                               the grid axis, the last tile of that axis is clipped to the grid
                               (a tile larger than the axis is the whole axis)                */
  int32_t window[3];        /* window in TILES, the unit Algorithm 1 compares; >= 1          */
  int32_t center_mode;      /* VORTA_CENTER_*: how get_window_center_id treats border tiles  */
  int32_t bucket[3];        /* BCS bucket, the paper uses (2,3,2); border buckets are clipped;
                               at most 64 tokens after clipping to the grid                    */
  int32_t keep_num, keep_den; /* core-set ratio r = keep_num/keep_den, 0 < r <= 1 (paper: 1/2) */
  float softmax_scale;      /* <= 0 selects 1/sqrt(head_dim)                                 */
  int32_t rope_dims[3];     /* rotary position embedding of Q and K (section 3.3 names it as part of
                               the block and omits it from the equations; the axial 3-D form is this
                               library's reading): the first rope_dims[0] channels of a head turn with
                               the token's frame index, the next rope_dims[1] with its row, the next
                               rope_dims[2] with its column; channels (2i, 2i+1) of an axis' span s
                               turn by position * rope_theta^(-2i / s).  Even, >= 0, sum <= head_dim;
                               channels beyond the sum and text tokens do not turn.  All zero: the
                               caller's q and k are used as they are (no RoPE, or already applied --
                               which is only right if no head takes route 2, see below).           */
  float rope_theta;         /* <= 0 selects 10000                                             */
} vorta_layer_desc;

typedef struct vorta_plan vorta_plan;   /* opaque */

typedef struct vorta_plan_info {
  int64_t n_video;          /* L                                                             */
  int64_t n_tokens;         /* N = L + n_text                                                */
  int32_t tiles[3];         /* tile grid n = ceil(grid / tile)                               */
  int32_t n_tiles;
  int32_t tile_tokens;      /* tokens of a full (unclipped) tile                             */
  int32_t window_key_tiles; /* key tiles every video query sees (clamp mode; max otherwise)  */
  int32_t max_runs;         /* row stride of the window run table                            */
  int32_t n_buckets;
  int64_t n_core;           /* L_c: core-set slots of the video tokens                       */
  int64_t n_core_tokens;    /* L_c + n_text: rows of a core-set buffer                       */
  int32_t elem_bytes;
} vorta_plan_info;

const char* vorta_strerror(int code);   /* static string                                       */
const char* vorta_last_error(void);     /* thread-local, valid until the thread's next call    */

/* ---- plan: host-side geometry of one layer ---------------------------------------------- */

/* Validates desc, builds the host index tables.  No HIP call.  *out is owned by the caller
 * and released with vorta_plan_destroy (which also frees the plan's device tables).
 * Size limit: (F*H*W + n_text) * row stride (head_dim, or heads * head_dim in the NHD layout)
 * must not exceed 2^31 elements -- rows are addressed with 32-bit element offsets -- else
 * VORTA_ESHAPE. */
int vorta_plan_create(const vorta_layer_desc* desc, vorta_plan** out);
int vorta_plan_destroy(vorta_plan* plan);

/* Set-up step for callers that want no allocation later: uploads the plan's index tables now
 * (blocking hipMalloc + hipMemcpy on the current device, which the plan then belongs to) instead
 * of on the first device call, and resolves the address of the library's static scratch on that
 * device.  Idempotent.  After it, no entry point allocates device memory for this plan. */
int vorta_plan_upload(vorta_plan* plan);

int vorta_plan_info_get(const vorta_plan* plan, vorta_plan_info* out);

/* ---- host tables: deterministic integers, checkable without a GPU ----------------------- */

/* Tile order (Algorithm 1's get_tile_id_3d made a storage order): token with raster index i
 * goes to position perm[i] = tile_row0[tile_id] + local_id, tile ids frame-major in the tile
 * grid, local ids frame-major inside the tile's own (possibly clipped) extents.  When the tile
 * divides the grid, tile_row0[t] = t * tile_tokens.  perm: host int32[L]. */
int vorta_tile_permutation(const vorta_plan* plan, int32_t* perm);

/* First tile-order row of every tile; tile t owns rows [tile_row0[t], tile_row0[t + 1]).
 * tile_row0: host int32[n_tiles + 1] (last entry = L). */
int vorta_tile_row0(const vorta_plan* plan, int32_t* tile_row0);

/* Algorithm 1 per query tile: the key tiles with abs(centre_d - k_d) <= window_d / 2 form
 * the box [lo_d, hi_d] (inclusive) returned as boxes[tile][6] = {loF,hiF,loH,hiH,loW,hiW}.
 * boxes: host int32[n_tiles][6]. */
int vorta_window_boxes(const vorta_plan* plan, int32_t* boxes);

/* The same boxes as runs of consecutive rows of a tile-ordered buffer, plus, if n_text > 0,
 * one run for the text rows: runs[tile][r] = {first_row, n_rows}, n_runs[tile] entries used.
 * runs: host int32[n_tiles][max_runs][2]; n_runs: host int32[n_tiles]. */
int vorta_window_runs(const vorta_plan* plan, int32_t* runs, int32_t* n_runs);

/* How the bf16 layer call cuts the work of route 1 (tiles of at most 128 tokens): query tiles
 * whose runs are identical see the same keys (Algorithm 1: under the clamped centre rule a border
 * tile and its inner neighbour on every axis, under the block rule all tiles of a block) and are
 * computed together, up to three tiles and 256 rows per work item.  items: host
 * int32[counts[0] + counts[1]][4] = {tile, tile, tile, n_tiles_in_item}, first the counts[0] items
 * of more than 128 rows, then the counts[1] items of at most 128 rows; every tile appears in
 * exactly one item.  items may be NULL to query the counts.  Both counts are 0 when a tile holds
 * more than 128 tokens (such tiles are cut into 256-row query blocks instead). */
int vorta_window_items(const vorta_plan* plan, int32_t* items, int32_t counts[2]);

/* BCS slot layout (section 3.2): buckets in raster order of bucket coordinates; bucket b owns
 * core-set slots [slot_base[b], slot_base[b+1]).  slot_base: host int32[n_buckets + 1]. */
int vorta_bcs_slot_bases(const vorta_plan* plan, int32_t* slot_base);

/* Eq. 4 bookkeeping: heads_by_route lists head ids grouped by route (route 0 first, ascending
 * id inside a group); counts[r] = heads on route r.  All host arrays. */
int vorta_route_partition(const vorta_plan* plan, const uint8_t* routes_host,
                          int32_t* heads_by_route, int32_t counts[3]);

/* Eq. 3: the router of one block, alpha = softmax(T W_R).  t_emb: host float[d_t], the
 * diffusion timestep embedding; w_r: host float[heads][d_t][3], one d_t x 3 projection per head
 * (the paper states one per block; per-head gates are what its per-head routing needs -- pass
 * the same matrix for every head to get per-block gates); alpha_out: host float[heads][3] =
 * (full, sliding, core-set), each row sums to 1.  Accumulation in double.  Returns
 * VORTA_EINVAL for null pointers or d_t < 1. */
int vorta_router_gates(const float* t_emb, const float* w_r, int32_t d_t, int32_t heads, float* alpha_out);

/* Eq. 4: gates alpha[heads][3] = (full, sliding, core-set) -> route codes; a branch is
 * taken only if its gate strictly exceeds both others, every tie goes to full.  Host arrays. */
int vorta_route_select(const float* alpha_host, int32_t heads, uint8_t* routes_host);

/* Eq. 3 and Eq. 4 on the device for a whole sampling schedule in one launch (the gates depend on
 * the timestep embedding only, section 3.3 "Attention router", so the routes of every step can be
 * had before sampling starts).  t_emb: device float[n_steps][d_t]; w_r: device
 * float[heads][d_t][3]; alpha: device float[n_steps][heads][3] (out); routes: device
 * uint8[n_steps][heads] (out).  Logits, softmax and the comparison of Eq. 4 are fp64 (ties go to
 * full attention), the gates are stored rounded to fp32.  routes_host, if not NULL, receives a
 * copy of `routes` through an asynchronous device-to-host copy on `stream` (pinned host memory
 * keeps it asynchronous): synchronise the stream before reading it -- the layer call takes its
 * routes from the host.  n_steps <= 65535.  Allocates nothing. */
int vorta_router_device(const float* t_emb, const float* w_r, int32_t n_steps, int32_t d_t, int32_t heads,
                        float* alpha, uint8_t* routes, uint8_t* routes_host, void* stream);

/* ---- device passes ------------------------------------------------------------------------ */

/* Token reorder, raster order -> tile order, for the heads on route 1 (Algorithm 1 needs
 * tile-contiguous tokens for a block-dense mask).  src: user layout.  dst: [n_win][N][d]
 * (slot-major; text rows copied unchanged after the L video rows). */
int vorta_reorder_to_tiles(vorta_plan* plan, const void* src, const uint8_t* routes_host,
                           void* dst, void* stream);

/* Inverse: src [n_win][N][d] in tile order -> rows of the route-1 heads of dst (user layout,
 * raster order).  Rows of other heads are not touched. */
int vorta_reorder_from_tiles(vorta_plan* plan, const void* src, const uint8_t* routes_host,
                             void* dst, void* stream);

/* Bucketed core-set selection for the heads on route 2 (section 3.2, Fig. 3).  feat: the feature
 * the similarity is taken on, head_dim elements per token.  feat_head_stride says how it is laid
 * out: VORTA_FEAT_USER_LAYOUT = a tensor in the user layout (the layer call passes K this way);
 * 0 = ONE array [L][head_dim] shared by every head (the core-set equation pools the block's
 * input, which has no head axis: all heads then select the same tokens); s > 0 = [heads][.][head_dim]
 * with s >= L * head_dim elements from one head to the next.  Per bucket: cosine similarity (fp64) of
 * the centre token to every other token, the k = floor(B (1 - r)) most similar are pruned
 * (ties: smaller local raster index first).  Outputs, slot-major:
 *   keep_idx int32[n_lr][L_c]  raster index of the token in each core-set slot
 *   assign   int32[n_lr][L]    slot each token reads its output from (own slot if kept,
 *                              its bucket centre's slot if pruned). */
#define VORTA_FEAT_USER_LAYOUT (-1)
int vorta_bcs_build_index(vorta_plan* plan, const void* feat, int64_t feat_head_stride,
                          const uint8_t* routes_host, int32_t* keep_idx, int32_t* assign, void* stream);

/* pool(): dst[slot][s] = mean of src rows assigned to core-set slot s (a kept token alone,
 * or a centre with the tokens pruned into it), then the text rows unchanged.  src: user
 * layout; dst: [n_lr][L_c + n_text][d].  Call once per tensor (Q, K, V).
 * rotate != 0 (for Q and K of a plan with rope_dims): the pooled row is then turned by the
 * rotary embedding at the position of the token that owns the slot, keep_idx[s] -- pooling
 * acts on the block's input and commutes with the projections but not with RoPE, so on route 2
 * the rotation comes after pool(); mean and rotation are computed in fp64 and rounded once. */
int vorta_bcs_pool(vorta_plan* plan, const void* src, const uint8_t* routes_host,
                   const int32_t* keep_idx, const int32_t* assign, int32_t rotate, void* dst, void* stream);

/* vorta_bcs_build_index on K followed by vorta_bcs_pool of Q, K (rotate = 1) and V, as ONE pass
 * over the data where the plan allows it (buckets of at most 16 tokens, rows of 256 bytes: the
 * paper's (2,3,2) bucket in bf16) -- K is then read from memory once and all rows of a bucket are
 * requested together; otherwise the four separate passes.  The results are those of the separate
 * calls, bit for bit.  This is the form the layer call runs (section 3.2: selection and merging
 * are both O(L), appendix complexity paragraph). */
int vorta_bcs_select_pool(vorta_plan* plan, const void* q, const void* k, const void* v,
                          const uint8_t* routes_host, int32_t* keep_idx, int32_t* assign, void* q_c, void* k_c,
                          void* v_c, void* stream);

/* Rotary embedding for the heads on routes 0 and 1: dst rows of those heads = src rows turned
 * at their token's grid position (text rows copied).  src, dst: user layout (dst rows of other
 * heads are not touched); a no-op returning VORTA_OK when the plan has no rope_dims.  The layer
 * call runs it on Q and K; route 2 rotates inside vorta_bcs_pool instead. */
int vorta_rope_apply(vorta_plan* plan, const void* src, const uint8_t* routes_host, void* dst, void* stream);

/* Buffers of the fused attention launch.  Unused groups may be NULL when no head takes
 * that route.  bf16 only: q_t, k_t, v_t and o_t may ALL be NULL although heads take route 1 --
 * the window kernel then gathers the rows of q, k, v through the tile permutation and writes
 * its output rows straight to their places in `out` (no tile-ordered copies, no reorder
 * passes); vorta_scatter_back is then called with o_t = NULL.  This is what the layer call does. */
typedef struct vorta_attn_io {
  const void *q, *k, *v;        /* user layout; read by route-0 heads (q, k as attention is to see
                                   them: after vorta_rope_apply if the plan has rope_dims)      */
  void* out;                    /* user layout; route-0 heads write their rows here            */
  const void *q_t, *k_t, *v_t;  /* [n_win][N][d] tile order (vorta_reorder_to_tiles)           */
  void* o_t;                    /* [n_win][N][d] tile order                                    */
  const void *q_c, *k_c, *v_c;  /* [n_lr][L_c + n_text][d] (vorta_bcs_pool)                    */
  void* o_c;                    /* [n_lr][L_c + n_text][d]                                     */
} vorta_attn_io;

/* softmax(scale * Q K^T) V for every head in one call: route 0 over all N keys (Eq. 2),
 * route 1 over the key tiles of vorta_window_runs plus text keys (Algorithm 1), route 2
 * over the pooled core-set rows.  bf16: MFMA contractions, fp32 softmax statistics, P and
 * the output rounded to bf16.  fp32: fp32 throughout. */
int vorta_attention_routed(vorta_plan* plan, const uint8_t* routes_host,
                           const vorta_attn_io* io, void* stream);

/* Back to sequence order (section 3.2: the sliding-tile branch computes on tile-contiguous
 * tokens, the core-set branch ends with unpool()): route 1 rows by the inverse tile permutation
 * from o_t (bf16 only: skipped when o_t is NULL, see vorta_attn_io; with fp32 a NULL o_t while
 * heads take route 1 is VORTA_EINVAL), route 2 rows by unpool() -- out[i] = o_c[assign[i]], text
 * rows from o_c[L_c + t] -- into the user-layout out.  Route 0 rows are already in place. */
int vorta_scatter_back(vorta_plan* plan, const uint8_t* routes_host, const void* o_t,
                       const void* o_c, const int32_t* assign, void* out, void* stream);

/* ---- the whole path ----------------------------------------------------------------------- */

/* Bytes of device scratch the layer call needs for these routes (internal buffers above; with
 * bf16 the four tile-ordered buffers are empty because the layer call does not make them). */
int vorta_workspace_bytes(const vorta_plan* plan, const uint8_t* routes_host, size_t* bytes);

/* Byte offsets of the internal buffers inside the workspace, in the order
 * q_t,k_t,v_t,o_t,q_c,k_c,v_c,o_c,keep_idx,assign,q_r,k_r (for inspection by tests); q_r and
 * k_r are the rotated copies of Q and K (user layout, empty without rope_dims). */
int vorta_workspace_layout(const vorta_plan* plan, const uint8_t* routes_host, size_t offsets[12]);

/* One attention layer under hard routing (Eq. 4; section 3.3 "Inference-time routing
 * strategy"): every head runs the branch its route names -- Eq. 2, Algorithm 1 or the core-set
 * branch of section 3.2.  reorder + index build + pool + fused attention + scatter back, all on
 * `stream`: q, k, v (user layout) -> out (user layout).  The BCS feature is K.  With rope_dims,
 * q and k are the projections BEFORE the rotary embedding: routes 0 and 1 attend on rotated
 * copies, route 2 selects and pools on the rows as given and rotates the pooled rows. */
int vorta_routed_attention_layer(vorta_plan* plan, const void* q, const void* k, const void* v,
                                 const uint8_t* routes_host, void* out, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* Eq. 5 (router optimisation forward): every head runs all three branches and the outputs
 * are blended with its gates, out = a1 attn + a2 sliding + a3 coreset.  alpha_host:
 * host float[heads][3].  workspace: vorta_soft_mixture_workspace_bytes.
 * bf16: fused -- the core-set branch leaves its pooled output rows in the workspace, the
 * sliding-tile branch writes the video rows of `out`, and the epilogue of the full-attention
 * branch reads both and writes the gate-weighted sum (fp32 arithmetic, one rounding to bf16 on
 * top of each branch's own); no branch is stored in full and there is no blend pass.  The
 * workspace is that of a layer whose heads all take route 2.  fp32: three full outputs in the
 * workspace and a blend pass. */
int vorta_soft_mixture_workspace_bytes(const vorta_plan* plan, size_t* bytes);
int vorta_soft_mixture_layer(vorta_plan* plan, const void* q, const void* k, const void* v,
                             const float* alpha_host, void* out, void* workspace,
                             size_t workspace_bytes, void* stream);

/* ---- for callers that cannot allocate ------------------------------------------------------- */

/* vorta_routed_attention_layer without a workspace argument and without any allocation, for
 * callers that must not call hipMalloc: code under HIP graph capture, tight serving loops,
 * harnesses that forbid it.  The internal buffers live in a fixed array of
 * VORTA_STATIC_SCRATCH_BYTES inside the library's device image (every GPU the library runs on
 * holds one until the process ends).  Requirements: vorta_plan_upload(plan) has been called (else
 * VORTA_EINVAL -- this call never uploads), and vorta_workspace_bytes(plan, routes) fits the
 * array (else VORTA_EWORKSPACE).  All calls on one GPU share the array: two calls whose stream
 * work overlaps in time race; calls on one stream are ordered.  Nothing in the array needs to
 * start at zero -- every buffer is fully written before it is read.  Results are those of
 * vorta_routed_attention_layer, bit for bit. */
#define VORTA_STATIC_SCRATCH_BYTES (32u << 20)
int vorta_routed_attention_layer_static(vorta_plan* plan, const void* q, const void* k, const void* v,
                                        const uint8_t* routes_host, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VORTA_H */
