// Memory-bound passes of the routed attention layer for gfx950: token reorder to / from
// 3-D tile order, bucketed core-set selection (index build), pool / merge, unpool, and the
// gate-weighted blend of Eq. 5.  All of them move 16-byte chunks of token rows (a 256-byte
// bf16 row of head_dim 128 is one fully coalesced segment whatever order rows are visited in);
// the index arithmetic is done once per row chunk and amortised over the heads of a route.
#include <hip/hip_runtime.h>

#include <cstring>

#include "vorta_internal.h"

namespace vorta {

#define VORTA_HIP(call)                                                                    \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess) return fail(VORTA_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

static int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(VORTA_EHIP, "launch of %s: %s", what, hipGetErrorString(e));
  return VORTA_OK;
}

// Uploads one host table; the device pointer is registered in *slot before the copy so that a
// failure anywhere leaves it for release_device_tables.
template <typename T>
static int upload_table(const std::vector<T>& host, T** slot) {
  VORTA_HIP(hipMalloc(slot, host.size() * sizeof(T)));
  VORTA_HIP(hipMemcpy(*slot, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  return VORTA_OK;
}

static void release_device_tables(vorta_plan* p) {
  int32_t** tables[] = {&p->d_runs, &p->d_n_runs, &p->d_slot_base, &p->d_tok_of, &p->d_tile_row0};
  for (int32_t** t : tables) {
    if (*t) (void)hipFree(*t);
    *t = nullptr;
  }
  if (p->d_rope_cs) (void)hipFree(p->d_rope_cs);
  p->d_rope_cs = nullptr;
  if (p->d_win_items) (void)hipFree(p->d_win_items);
  p->d_win_items = nullptr;
}
// vorta_plan_destroy lives with the host code; it frees the device tables through this hook
static const bool release_hook_set = (g_release_device_tables = release_device_tables, true);

static int upload_device_tables(vorta_plan* p, int dev) {
  if (int rc = upload_table(p->runs, &p->d_runs)) return rc;
  if (int rc = upload_table(p->n_runs, &p->d_n_runs)) return rc;
  if (int rc = upload_table(p->slot_base, &p->d_slot_base)) return rc;
  if (int rc = upload_table(p->tile_row0, &p->d_tile_row0)) return rc;
  // tile-order row -> token (the inverse tile permutation; text rows keep their place)
  std::vector<int32_t> perm((size_t)p->L), tok_of((size_t)p->N);
  if (int rc = vorta_tile_permutation(p, perm.data())) return rc;
  for (int64_t i = 0; i < p->L; ++i) tok_of[perm[i]] = (int32_t)i;
  for (int64_t i = p->L; i < p->N; ++i) tok_of[i] = (int32_t)i;
  if (int rc = upload_table(tok_of, &p->d_tok_of)) return rc;
  if (p->rope)
    if (int rc = upload_table(p->rope_cs, &p->d_rope_cs)) return rc;
  if (!p->win_items.empty())
    if (int rc = upload_table(p->win_items, &p->d_win_items)) return rc;
  int cus = 0;
  VORTA_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (cus > 0) p->n_cus = cus;
  return VORTA_OK;
}

int ensure_device_tables(vorta_plan* p) {
  std::lock_guard<std::mutex> lock(p->mu);
  int dev = -1;
  VORTA_HIP(hipGetDevice(&dev));
  if (p->on_device) {
    // the tables live on the device that was current at the plan's first device call
    if (dev != p->device)
      return fail(VORTA_EINVAL, "plan belongs to device %d, current device is %d: one plan per device", p->device, dev);
    return VORTA_OK;
  }
  if (int rc = upload_device_tables(p, dev)) {
    release_device_tables(p);      // nothing half-built is kept; the next call starts over
    return rc;
  }
  p->device = dev;
  p->on_device = true;
  return VORTA_OK;
}

struct HeadList {
  int n;
  uint8_t id[VORTA_MAX_HEADS];
};

static HeadList head_list(const RouteLists& rl, int route) {
  HeadList h;
  h.n = rl.count[route];
  for (int i = 0; i < h.n; ++i) h.id[i] = (uint8_t)rl.heads[route][i];
  return h;
}

struct Geo {
  int F, H, W;
  int L, N;
  int bF, bH, bW;   // bucket
  int nbH, nbW;     // bucket grid along H, W
  int keep_num, keep_den;
};

static Geo make_geo(const vorta_plan* p) {
  Geo g;
  g.F = p->d.F; g.H = p->d.H; g.W = p->d.W;
  g.L = (int)p->L; g.N = (int)p->N;
  g.bF = p->d.bucket[0]; g.bH = p->d.bucket[1]; g.bW = p->d.bucket[2];
  g.nbH = p->nb[1]; g.nbW = p->nb[2];
  g.keep_num = p->d.keep_num; g.keep_den = p->d.keep_den;
  return g;
}

// Rotary embedding: the table holds (cos, sin) per position and channel pair, axis after axis.
struct Rope {
  const float2* cs;     // [F][pF], [H][pH], [W][pW]
  int pF, pH, pW;       // channel pairs that turn with the frame index, the row, the column
  int baseH, baseW;     // first table entry of the H and W axes
  int H, W;             // grid extents, to decode a token index
};

static Rope make_rope(const vorta_plan* p) {
  Rope r;
  r.cs = (const float2*)p->d_rope_cs;
  r.pF = p->d.rope_dims[0] / 2; r.pH = p->d.rope_dims[1] / 2; r.pW = p->d.rope_dims[2] / 2;
  r.baseH = p->d.F * r.pF;
  r.baseW = r.baseH + p->d.H * r.pH;
  r.H = p->d.H; r.W = p->d.W;
  return r;
}

// Turns the NP channel pairs x[2i], x[2i+1] that start at channel pair `pair0` of the head,
// for the video token `tok`.  Pairs past the three spans are left alone.
template <int NP>
__device__ __forceinline__ void rope_turn(const Rope& r, int tok, int pair0, double* x) {
#pragma clang fp contract(off)
  const int hw = r.H * r.W;
  const int f = tok / hw, rem = tok - f * hw;
  const int h = rem / r.W, w = rem - h * r.W;
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int j = pair0 + i;
    int idx = -1;
    if (j < r.pF) idx = f * r.pF + j;
    else if (j < r.pF + r.pH) idx = r.baseH + h * r.pH + (j - r.pF);
    else if (j < r.pF + r.pH + r.pW) idx = r.baseW + w * r.pW + (j - r.pF - r.pH);
    if (idx >= 0) {
      const float2 cs = r.cs[idx];
      const double a = x[2 * i], b = x[2 * i + 1];
      x[2 * i] = a * (double)cs.x - b * (double)cs.y;
      x[2 * i + 1] = a * (double)cs.y + b * (double)cs.x;
    }
  }
}

// ------------------------------------------------------------------------------------------
// reorder: one thread per (tile-order row, 16-byte chunk), looping over the heads of route 1
// ------------------------------------------------------------------------------------------
template <bool TO_TILES>
__global__ __launch_bounds__(256) void reorder_kernel(uint4* __restrict__ user, uint4* __restrict__ tiled,
                                                      const int* __restrict__ tok_of, HeadList hl, int N,
                                                      long head_stride_c, long row_stride_c, int cshift) {
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const int pos = (int)(gid >> cshift);
  const int c = (int)(gid & ((1 << cshift) - 1));
  if (pos >= N) return;
  const int i = tok_of[pos];   // tile-order row -> token (text rows keep their place)
  const long u0 = (long)i * row_stride_c + c;
  const long t0 = ((long)pos << cshift) + c;
  const long tiled_head = (long)N << cshift;
#pragma unroll 4
  for (int s = 0; s < hl.n; ++s) {
    const long u = u0 + hl.id[s] * head_stride_c, t = t0 + s * tiled_head;
    if (TO_TILES) tiled[t] = user[u];
    else user[u] = tiled[t];
  }
}

static int chunk_shift(const vorta_plan* p) {
  const int chunks = p->d.head_dim * p->elem_bytes / 16;   // 16 or 32
  return chunks == 32 ? 5 : 4;
}

int launch_reorder(vorta_plan* p, const RouteLists& rl, const void* user, void* tiled, bool to_tiles,
                   void* stream) {
  if (rl.count[1] == 0) return VORTA_OK;
  const UserTensor ut = user_tensor(p, user);
  const int cs = chunk_shift(p);
  const int epc = 16 / p->elem_bytes;   // elements per chunk
  const long total = (long)p->N << cs;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  const HeadList hl = head_list(rl, 1);
  hipStream_t st = (hipStream_t)stream;
  if (to_tiles)
    hipLaunchKernelGGL(reorder_kernel<true>, dim3(blocks), dim3(256), 0, st, (uint4*)user, (uint4*)tiled,
                       p->d_tok_of, hl, (int)p->N, ut.head_stride / epc, ut.row_stride / epc, cs);
  else
    hipLaunchKernelGGL(reorder_kernel<false>, dim3(blocks), dim3(256), 0, st, (uint4*)user, (uint4*)tiled,
                       p->d_tok_of, hl, (int)p->N, ut.head_stride / epc, ut.row_stride / epc, cs);
  return launch_status("reorder_kernel");
}

// ------------------------------------------------------------------------------------------
// unpool: out[i] = o_c[assign[i]] for the heads of route 2 (text rows: o_c[L_c + t])
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void unpool_kernel(uint4* __restrict__ out, const uint4* __restrict__ o_c,
                                                     const int* __restrict__ assign, HeadList hl, int L,
                                                     int N, int Lc, long head_stride_c, long row_stride_c,
                                                     int cshift) {
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const int i = (int)(gid >> cshift);
  const int c = (int)(gid & ((1 << cshift) - 1));
  if (i >= N) return;
  const long u0 = (long)i * row_stride_c + c;
  const long core_head = (long)(Lc + N - L) << cshift;
#pragma unroll 4
  for (int s = 0; s < hl.n; ++s) {
    const int slot = i < L ? assign[(long)s * L + i] : Lc + (i - L);
    out[u0 + hl.id[s] * head_stride_c] = o_c[s * core_head + ((long)slot << cshift) + c];
  }
}

int launch_unpool(vorta_plan* p, const RouteLists& rl, const void* o_c, const int32_t* assign, void* out,
                  void* stream) {
  if (rl.count[2] == 0) return VORTA_OK;
  const UserTensor ut = user_tensor(p, out);
  const int cs = chunk_shift(p);
  const int epc = 16 / p->elem_bytes;
  const long total = (long)p->N << cs;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(unpool_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)out,
                     (const uint4*)o_c, assign, head_list(rl, 2), (int)p->L, (int)p->N, (int)p->Lc,
                     ut.head_stride / epc, ut.row_stride / epc, cs);
  return launch_status("unpool_kernel");
}

// ------------------------------------------------------------------------------------------
// Bucketed core-set selection (helpers; the kernels follow).
// ------------------------------------------------------------------------------------------
template <typename T> struct Elem;
template <> struct Elem<float> {
  __device__ static double load(const float* p) { return (double)*p; }
  __device__ static void store(float* p, double v) { *p = (float)v; }
};
template <> struct Elem<uint16_t> {   // bf16 bits
  __device__ static double load(const uint16_t* p) { return (double)__uint_as_float((unsigned)*p << 16); }
  __device__ static void store(uint16_t* p, double v) {
    const unsigned u = __float_as_uint((float)v);      // round-to-nearest-even on the upper 16 bits
    *p = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
  }
};

struct Bucket {
  int f0, h0, w0;   // origin
  int df, dh, dw;   // clipped extent
  int size, centre, prune;
};

__device__ __forceinline__ Bucket bucket_of(const Geo& g, int b) {
  Bucket k;
  const int per_f = g.nbH * g.nbW;
  const int bf = b / per_f, r = b - bf * per_f;
  const int bh = r / g.nbW, bw = r - bh * g.nbW;
  k.f0 = bf * g.bF; k.h0 = bh * g.bH; k.w0 = bw * g.bW;
  k.df = min(g.bF, g.F - k.f0); k.dh = min(g.bH, g.H - k.h0); k.dw = min(g.bW, g.W - k.w0);
  k.size = k.df * k.dh * k.dw;
  k.centre = ((k.df / 2) * k.dh + k.dh / 2) * k.dw + k.dw / 2;
  k.prune = min(k.size - 1, (int)(((long)k.size * (g.keep_den - g.keep_num)) / g.keep_den));
  return k;
}

__device__ __forceinline__ int bucket_token(const Geo& g, const Bucket& k, int j) {
  const int hw = k.dh * k.dw;
  const int a = j / hw, r = j - a * hw;
  const int b = r / k.dw, c = r - b * k.dw;
  return ((k.f0 + a) * g.H + k.h0 + b) * g.W + k.w0 + c;
}

// 16-byte chunk of a row (8 bf16 or 4 fp32 elements): raw load, and widening to fp64
template <typename T> struct Chunk;
template <> struct Chunk<uint16_t> {
  static constexpr int N = 8;
  __device__ static uint4 raw(const uint16_t* p) { return *(const uint4*)p; }
  __device__ static void widen(const uint4& u, double* x) {
    const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = (double)__uint_as_float(w[i] << 16);
      x[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static void load(const uint16_t* p, double* x) { widen(raw(p), x); }
};
template <> struct Chunk<float> {
  static constexpr int N = 4;
  __device__ static uint4 raw(const float* p) { return *(const uint4*)p; }
  __device__ static void widen(const uint4& u, double* x) {
    x[0] = __uint_as_float(u.x); x[1] = __uint_as_float(u.y); x[2] = __uint_as_float(u.z); x[3] = __uint_as_float(u.w);
  }
  __device__ static void load(const float* p, double* x) { widen(raw(p), x); }
};

// sum over the 4 lanes of a quad (lanes 4k .. 4k+3)
__device__ __forceinline__ double quad_sum(double v) {
  v += __shfl_xor(v, 1, 64);
  v += __shfl_xor(v, 2, 64);
  return v;
}

// One wavefront per (bucket, head).  Four lanes share a token: lane 4t + q holds quarter q of
// token t's feature row (16-byte loads, all rows of a pass in flight at once), so a pass of
// the wavefront covers 16 tokens; partial dot products and norms are fp64 and are summed
// over the quad.  Then lane j ranks token j.  The products are formed inside fused
// multiply-adds: a product of two bf16 (or fp32) values is exact in fp64, so fusing changes
// no bit and halves the fp64 instruction count; everything after the sums stays unfused.
// Cosine similarity of this quad's token to the bucket's centre from the lane's quarter rows
// (craw: centre, xraw: token).  nc, the centre's squared norm, is produced when first is set and
// reused afterwards.  Returns 0 for an invalid lane, a zero norm or a non-finite result.
template <typename T, int CH>
__device__ __forceinline__ double quad_similarity(const uint4 (&craw)[CH], const uint4 (&xraw)[CH], bool valid,
                                                  bool first, double& nc) {
#pragma clang fp contract(off)
  double dot = 0.0, nj = 0.0, ncp = 0.0;
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    double c[Chunk<T>::N], x[Chunk<T>::N];
    Chunk<T>::widen(craw[ch], c);
    Chunk<T>::widen(xraw[ch], x);
#pragma unroll
    for (int e = 0; e < Chunk<T>::N; ++e) {
      ncp = __builtin_fma(c[e], c[e], ncp);
      dot = __builtin_fma(c[e], x[e], dot);
      nj = __builtin_fma(x[e], x[e], nj);
    }
  }
  if (first) nc = quad_sum(ncp);
  dot = quad_sum(dot);
  nj = quad_sum(nj);
  double sim = 0.0;
  if (valid && nc != 0.0 && nj != 0.0) sim = dot / sqrt(nc * nj);
  if (!(sim == sim)) sim = 0.0;       // non-finite features: keep the ranking a total order
  return sim;
}

// Lane j holds the similarity of token j.  Ranks the non-centre tokens (larger similarity first,
// ties by index), prunes the first k.prune of them and numbers the kept tokens in raster order.
// Returns the slot token `lane` reads its output from (its own if kept, else the centre's);
// kept / own_slot say whether the lane's token owns a slot and which.
__device__ __forceinline__ int rank_and_assign(const Bucket& k, int lane, double my_sim, int base_slot, bool& kept,
                                               int& centre_slot) {
  int rank = 0;
  for (int m = 0; m < k.size; ++m) {
    const double sm = __shfl(my_sim, m, 64);
    if (m != k.centre && (sm > my_sim || (sm == my_sim && m < lane))) ++rank;
  }
  const bool in_bucket = lane < k.size;
  kept = in_bucket && (lane == k.centre || rank >= k.prune);
  const unsigned long long kept_mask = __ballot(kept);
  const int my_slot = base_slot + __popcll(kept_mask & ((1ull << lane) - 1ull));
  centre_slot = base_slot + __popcll(kept_mask & ((1ull << k.centre) - 1ull));
  return kept ? my_slot : centre_slot;
}

template <typename T, int D>   // D = head_dim
__global__ __launch_bounds__(256) void bcs_index_kernel(const T* __restrict__ feat, HeadList hl, Geo g,
                                                        int n_buckets, const int* __restrict__ slot_base,
                                                        long head_stride, long row_stride, int Lc,
                                                        int* __restrict__ keep_idx, int* __restrict__ assign) {
  constexpr int EP = D / 4;                 // elements per lane
  constexpr int CH = EP / Chunk<T>::N;      // 16-byte chunks per lane
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int s = blockIdx.y;
  if (b >= n_buckets) return;
  const Bucket k = bucket_of(g, b);
  const int quarter = lane & 3, tl = lane >> 2;
  const T* base = feat + hl.id[s] * head_stride + quarter * EP;

  // The centre row and the rows of the first pass are requested together; rows stay in their
  // 16-byte form and are widened chunk by chunk as they are used, so a bucket of up to 16
  // tokens costs one memory round trip.
  uint4 craw[CH];
  {
    const T* row = base + (long)bucket_token(g, k, k.centre) * row_stride;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) craw[ch] = Chunk<T>::raw(row + ch * Chunk<T>::N);
  }
  double nc = 0.0, my_sim = 0.0;
  for (int pass = 0; pass * 16 < k.size; ++pass) {
    const int j = pass * 16 + tl;
    const bool valid = j < k.size && j != k.centre;
    const T* row = base + (long)bucket_token(g, k, valid ? j : k.centre) * row_stride;
    uint4 xraw[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) xraw[ch] = Chunk<T>::raw(row + ch * Chunk<T>::N);
    const double sim = quad_similarity<T, CH>(craw, xraw, valid, pass == 0, nc);
    // token 16 pass + t sits in lanes 4t .. 4t+3; hand it to lane 16 pass + t
    const double mine = __shfl(sim, 4 * (lane & 15), 64);
    if ((lane >> 4) == pass) my_sim = mine;
  }

  bool kept;
  int centre_slot;
  const int slot = rank_and_assign(k, lane, my_sim, slot_base[b], kept, centre_slot);
  if (lane < k.size) {
    const int tok = bucket_token(g, k, lane);
    if (kept) keep_idx[(long)s * Lc + slot] = tok;
    assign[(long)s * g.L + tok] = slot;
  }
}

int launch_bcs_index(vorta_plan* p, const RouteLists& rl, const UserTensor& ut, int32_t* keep_idx,
                     int32_t* assign, void* stream) {
  if (rl.count[2] == 0) return VORTA_OK;
  const void* feat = ut.base;
  const dim3 grid((p->n_buckets + 3) / 4, rl.count[2]);
  const HeadList hl = head_list(rl, 2);
  const Geo g = make_geo(p);
  hipStream_t st = (hipStream_t)stream;
  if (p->d.dtype == VORTA_BF16)
    hipLaunchKernelGGL((bcs_index_kernel<uint16_t, 128>), grid, dim3(256), 0, st, (const uint16_t*)feat, hl, g,
                       p->n_buckets, p->d_slot_base, ut.head_stride, ut.row_stride, (int)p->Lc, keep_idx, assign);
  else if (p->d.head_dim == 64)
    hipLaunchKernelGGL((bcs_index_kernel<float, 64>), grid, dim3(256), 0, st, (const float*)feat, hl, g,
                       p->n_buckets, p->d_slot_base, ut.head_stride, ut.row_stride, (int)p->Lc, keep_idx, assign);
  else
    hipLaunchKernelGGL((bcs_index_kernel<float, 128>), grid, dim3(256), 0, st, (const float*)feat, hl, g,
                       p->n_buckets, p->d_slot_base, ut.head_stride, ut.row_stride, (int)p->Lc, keep_idx, assign);
  return launch_status("bcs_index_kernel");
}

// ------------------------------------------------------------------------------------------
// pool / merge: one wavefront per (bucket, head).  A row is CPR 16-byte chunks; lane
// (c = lane % CPR, group = lane / CPR) moves chunk c of the tokens group, group + G, ...
// (G = 64 / CPR token groups).  A kept token's chunk is copied to its slot; the chunks of the
// centre and of the tokens pruned into it are summed in fp64, the G partial sums are added
// across the groups, and group 0 writes the mean to the centre's slot.
// ------------------------------------------------------------------------------------------
// ROPE: every pooled row is turned by the rotary embedding at the position of the token that owns
// its slot (the kept token itself; for a merged row the bucket's centre) before it is stored.
template <typename T, int D, bool ROPE>
__global__ __launch_bounds__(256) void bcs_pool_kernel(const T* __restrict__ src, HeadList hl, Geo g,
                                                       int n_buckets, long head_stride, long row_stride,
                                                       int n_core_rows, const int* __restrict__ assign,
                                                       T* __restrict__ dst, Rope rope) {
  constexpr int CN = Chunk<T>::N;           // elements per chunk
  constexpr int CPR = D / CN;               // chunks per row: 16 or 32
  constexpr int G = 64 / CPR;               // token groups per pass
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int s = blockIdx.y;
  if (b >= n_buckets) return;
  const Bucket k = bucket_of(g, b);
  const int c = lane % CPR, grp = lane / CPR;
  const T* base = src + hl.id[s] * head_stride + c * CN;
  T* out = dst + (long)s * n_core_rows * D + c * CN;

  int my_slot = 0;
  if (lane < k.size) my_slot = assign[(long)s * g.L + bucket_token(g, k, lane)];
  const int centre_slot = __shfl(my_slot, k.centre, 64);
  double acc[CN];
#pragma unroll
  for (int e = 0; e < CN; ++e) acc[e] = 0.0;
  int members = 0;
  for (int j0 = 0; j0 < k.size; j0 += G) {
    const int j = j0 + grp;
    const int slot = __shfl(my_slot, min(j, k.size - 1), 64);
    // members of the centre's cluster among the G tokens of this pass (same count in every lane)
#pragma unroll
    for (int q = 0; q < G; ++q)
      if (j0 + q < k.size && __shfl(my_slot, min(j0 + q, k.size - 1), 64) == centre_slot) ++members;
    if (j >= k.size) continue;
    const int tok = bucket_token(g, k, j);
    const T* row = base + (long)tok * row_stride;
    if (slot == centre_slot) {
      double x[CN];
      Chunk<T>::load(row, x);
#pragma unroll
      for (int e = 0; e < CN; ++e) acc[e] += x[e];
    } else if (ROPE) {
      double x[CN];
      Chunk<T>::load(row, x);
      rope_turn<CN / 2>(rope, tok, c * (CN / 2), x);
      T* o = out + (long)slot * D;
#pragma unroll
      for (int e = 0; e < CN; ++e) Elem<T>::store(o + e, x[e]);
    } else {
      *(uint4*)(out + (long)slot * D) = *(const uint4*)row;
    }
  }
#pragma unroll
  for (int e = 0; e < CN; ++e) {
    double v = acc[e];
#pragma unroll
    for (int off = CPR; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
    acc[e] = v / (double)members;
  }
  if (ROPE) rope_turn<CN / 2>(rope, bucket_token(g, k, k.centre), c * (CN / 2), acc);
  if (grp == 0) {
    T* o = out + (long)centre_slot * D;
#pragma unroll
    for (int e = 0; e < CN; ++e) Elem<T>::store(o + e, acc[e]);
  }
}

// text rows ride along unchanged behind the L_c pooled rows
__global__ __launch_bounds__(256) void copy_text_rows_kernel(const uint4* __restrict__ user,
                                                             uint4* __restrict__ core, HeadList hl, int L,
                                                             int n_text, int Lc, long head_stride_c,
                                                             long row_stride_c, int cshift) {
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const int t = (int)(gid >> cshift);
  const int c = (int)(gid & ((1 << cshift) - 1));
  if (t >= n_text) return;
  const long core_head = (long)(Lc + n_text) << cshift;
  for (int s = 0; s < hl.n; ++s)
    core[s * core_head + ((long)(Lc + t) << cshift) + c] =
        user[hl.id[s] * head_stride_c + (long)(L + t) * row_stride_c + c];
}

int launch_bcs_pool(vorta_plan* p, const RouteLists& rl, const void* src, const int32_t* keep_idx,
                    const int32_t* assign, bool rotate, void* dst, void* stream) {
  (void)keep_idx;   // the slot of every token is in `assign`; kept for a symmetric interface
  if (rl.count[2] == 0) return VORTA_OK;
  const UserTensor ut = user_tensor(p, src);
  const dim3 grid((p->n_buckets + 3) / 4, rl.count[2]);
  const HeadList hl = head_list(rl, 2);
  const Geo g = make_geo(p);
  const int rows = (int)(p->Lc + p->d.n_text);
  hipStream_t st = (hipStream_t)stream;
  const bool rope_on = rotate && p->rope;
  const Rope rope = make_rope(p);
#define VORTA_POOL(T_, D_, R_)                                                                                  \
  hipLaunchKernelGGL((bcs_pool_kernel<T_, D_, R_>), grid, dim3(256), 0, st, (const T_*)src, hl, g, p->n_buckets, \
                     ut.head_stride, ut.row_stride, rows, assign, (T_*)dst, rope)
  if (p->d.dtype == VORTA_BF16) {
    if (rope_on) VORTA_POOL(uint16_t, 128, true); else VORTA_POOL(uint16_t, 128, false);
  } else if (p->d.head_dim == 64) {
    if (rope_on) VORTA_POOL(float, 64, true); else VORTA_POOL(float, 64, false);
  } else {
    if (rope_on) VORTA_POOL(float, 128, true); else VORTA_POOL(float, 128, false);
  }
#undef VORTA_POOL
  if (int rc = launch_status("bcs_pool_kernel")) return rc;
  if (p->d.n_text > 0) {
    const int cs = chunk_shift(p);
    const int epc = 16 / p->elem_bytes;
    const long total = (long)p->d.n_text << cs;
    hipLaunchKernelGGL(copy_text_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const uint4*)src, (uint4*)dst, hl, (int)p->L, p->d.n_text, (int)p->Lc,
                       ut.head_stride / epc, ut.row_stride / epc, cs);
    return launch_status("copy_text_rows_kernel");
  }
  return VORTA_OK;
}

// ------------------------------------------------------------------------------------------
// Select and pool in one pass (what the layer call runs when a bucket holds at most 16 tokens and
// a row is 16 chunks, which covers the paper's (2,3,2) bucket in bf16): one wavefront per (bucket,
// head) requests, before it computes anything, the bucket's K rows in the index kernel's form (a
// quarter row per lane) and its Q, K and V rows in the pool kernel's form (chunk c of tokens grp,
// grp + 4, ...), so one memory round trip covers them all and K comes from HBM once; then it
// ranks exactly as bcs_index_kernel does, writes keep_idx / assign, and merges and stores the
// three tensors exactly as bcs_pool_kernel does (same operations in the same order: the results
// of the two forms are identical bit for bit).
// ------------------------------------------------------------------------------------------
template <typename T, int D, bool ROPE>
__global__ __launch_bounds__(256) void bcs_select_pool_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                              const T* __restrict__ v, HeadList hl, Geo g, int n_buckets,
                                                              const int* __restrict__ slot_base, long head_stride,
                                                              long row_stride, int Lc, int n_core_rows,
                                                              int* __restrict__ keep_idx, int* __restrict__ assign,
                                                              T* __restrict__ qc, T* __restrict__ kc, T* __restrict__ vc,
                                                              Rope rope) {
  constexpr int CN = Chunk<T>::N;
  static_assert(D / CN == 16, "rows of 16 chunks");
  constexpr int EP = D / 4, CH = EP / CN;   // index form: elements and chunks per lane
  constexpr int G = 4, P = 4;               // pool form: token groups per pass, passes for up to 16 tokens
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int s = blockIdx.y;
  if (b >= n_buckets) return;
  const Bucket kb = bucket_of(g, b);        // kb.size <= 16: checked on the host
  const long head_off = hl.id[s] * head_stride;

  // ---- every load of the wavefront
  const int quarter = lane & 3, tl = lane >> 2;
  const bool valid = tl < kb.size && tl != kb.centre;
  uint4 craw[CH], xraw[CH];
  {
    const T* crow = k + head_off + (long)bucket_token(g, kb, kb.centre) * row_stride + quarter * EP;
    const T* xrow = k + head_off + (long)bucket_token(g, kb, valid ? tl : kb.centre) * row_stride + quarter * EP;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      craw[ch] = Chunk<T>::raw(crow + ch * CN);
      xraw[ch] = Chunk<T>::raw(xrow + ch * CN);
    }
  }
  const int c = lane & 15, grp = lane >> 4;
  uint4 rq[P], rk[P], rv[P];
  int tok_p[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    tok_p[p] = bucket_token(g, kb, min(G * p + grp, kb.size - 1));
    const long off = head_off + (long)tok_p[p] * row_stride + c * CN;
    rq[p] = Chunk<T>::raw(q + off);
    rk[p] = Chunk<T>::raw(k + off);
    rv[p] = Chunk<T>::raw(v + off);
  }

  // ---- select
  double nc = 0.0;
  const double sim = quad_similarity<T, CH>(craw, xraw, valid, true, nc);
  const double mine = __shfl(sim, 4 * (lane & 15), 64);
  const double my_sim = lane < 16 ? mine : 0.0;
  bool kept;
  int centre_slot;
  const int slot_of_lane = rank_and_assign(kb, lane, my_sim, slot_base[b], kept, centre_slot);
  if (lane < kb.size) {
    const int tok = bucket_token(g, kb, lane);
    if (kept) keep_idx[(long)s * Lc + slot_of_lane] = tok;
    assign[(long)s * g.L + tok] = slot_of_lane;
  }

  // ---- pool
  const int centre_tok = bucket_token(g, kb, kb.centre);
  const int members = kb.prune + 1;
  int slot_p[P];
#pragma unroll
  for (int p = 0; p < P; ++p) slot_p[p] = __shfl(slot_of_lane, min(G * p + grp, kb.size - 1), 64);
  auto pool = [&](const uint4 (&rows)[P], T* dst, bool rotate) {
    T* out = dst + (long)s * n_core_rows * D + c * CN;
    double acc[CN];
#pragma unroll
    for (int e = 0; e < CN; ++e) acc[e] = 0.0;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      if (G * p + grp >= kb.size) continue;
      if (slot_p[p] == centre_slot) {
        double x[CN];
        Chunk<T>::widen(rows[p], x);
#pragma unroll
        for (int e = 0; e < CN; ++e) acc[e] += x[e];
      } else if (rotate) {
        double x[CN];
        Chunk<T>::widen(rows[p], x);
        rope_turn<CN / 2>(rope, tok_p[p], c * (CN / 2), x);
        T* o = out + (long)slot_p[p] * D;
#pragma unroll
        for (int e = 0; e < CN; ++e) Elem<T>::store(o + e, x[e]);
      } else {
        *(uint4*)(out + (long)slot_p[p] * D) = rows[p];
      }
    }
#pragma unroll
    for (int e = 0; e < CN; ++e) {
      double sum = acc[e];
      sum += __shfl_xor(sum, 16, 64);
      sum += __shfl_xor(sum, 32, 64);
      acc[e] = sum / (double)members;
    }
    if (rotate) rope_turn<CN / 2>(rope, centre_tok, c * (CN / 2), acc);
    if (grp == 0) {
      T* o = out + (long)centre_slot * D;
#pragma unroll
      for (int e = 0; e < CN; ++e) Elem<T>::store(o + e, acc[e]);
    }
  };
  pool(rq, qc, ROPE);
  pool(rk, kc, ROPE);
  pool(rv, vc, false);
}

// True when the fused form applies: buckets of at most 16 tokens, rows of 16 chunks.
bool bcs_fused_applies(const vorta_plan* p) {
  const long bucket_tokens = (long)p->d.bucket[0] * p->d.bucket[1] * p->d.bucket[2];
  const int chunks = p->d.head_dim * p->elem_bytes / 16;
  return bucket_tokens <= 16 && chunks == 16;
}

// Index on K, then Q, K, V pooled (Q and K rotated if the plan has a rotary embedding) into
// qc, kc, vc, and the text rows copied behind them.
int launch_bcs_select_pool(vorta_plan* p, const RouteLists& rl, const void* q, const void* k, const void* v,
                           int32_t* keep_idx, int32_t* assign, void* qc, void* kc, void* vc, void* stream) {
  if (rl.count[2] == 0) return VORTA_OK;
  const UserTensor ut = user_tensor(p, k);
  const dim3 grid((p->n_buckets + 3) / 4, rl.count[2]);
  const HeadList hl = head_list(rl, 2);
  const Geo g = make_geo(p);
  const int rows = (int)(p->Lc + p->d.n_text);
  const Rope rope = make_rope(p);
  hipStream_t st = (hipStream_t)stream;
#define VORTA_FUSED(T_, D_, R_)                                                                                        \
  hipLaunchKernelGGL((bcs_select_pool_kernel<T_, D_, R_>), grid, dim3(256), 0, st, (const T_*)q, (const T_*)k,         \
                     (const T_*)v, hl, g, p->n_buckets, p->d_slot_base, ut.head_stride, ut.row_stride, (int)p->Lc, rows, \
                     keep_idx, assign, (T_*)qc, (T_*)kc, (T_*)vc, rope)
  if (p->d.dtype == VORTA_BF16) {
    if (p->rope) VORTA_FUSED(uint16_t, 128, true); else VORTA_FUSED(uint16_t, 128, false);
  } else {
    if (p->rope) VORTA_FUSED(float, 64, true); else VORTA_FUSED(float, 64, false);
  }
#undef VORTA_FUSED
  if (int rc = launch_status("bcs_select_pool_kernel")) return rc;
  if (p->d.n_text > 0) {
    const int cs = chunk_shift(p);
    const int epc = 16 / p->elem_bytes;
    const long total = (long)p->d.n_text << cs;
    const void* srcs[3] = {q, k, v};
    void* dsts[3] = {qc, kc, vc};
    for (int t = 0; t < 3; ++t)
      hipLaunchKernelGGL(copy_text_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                         (const uint4*)srcs[t], (uint4*)dsts[t], hl, (int)p->L, p->d.n_text, (int)p->Lc,
                         ut.head_stride / epc, ut.row_stride / epc, cs);
    return launch_status("copy_text_rows_kernel");
  }
  return VORTA_OK;
}

// ------------------------------------------------------------------------------------------
// Rotary embedding of whole rows, heads of routes 0 and 1: one thread per (row, 16-byte chunk),
// looping over the heads; dst has the caller's layout.  Text rows are copied.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rope_rows_kernel(const T* __restrict__ src, T* __restrict__ dst, HeadList hl,
                                                        int L, int N, long head_stride, long row_stride, int cshift,
                                                        Rope rope) {
  constexpr int CN = Chunk<T>::N;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const int i = (int)(gid >> cshift);
  const int c = (int)(gid & ((1 << cshift) - 1));
  if (i >= N) return;
  const long off0 = (long)i * row_stride + c * CN;
#pragma unroll 2
  for (int s = 0; s < hl.n; ++s) {
    const long off = off0 + hl.id[s] * head_stride;
    if (i >= L) {
      *(uint4*)(dst + off) = *(const uint4*)(src + off);
      continue;
    }
    double x[CN];
    Chunk<T>::load(src + off, x);
    rope_turn<CN / 2>(rope, i, c * (CN / 2), x);
#pragma unroll
    for (int e = 0; e < CN; ++e) Elem<T>::store(dst + off + e, x[e]);
  }
}

int launch_rope_rows(vorta_plan* p, const RouteLists& rl, const void* src, void* dst, void* stream) {
  HeadList hl;
  hl.n = 0;
  for (int r = 0; r < 2; ++r)
    for (int i = 0; i < rl.count[r]; ++i) hl.id[hl.n++] = (uint8_t)rl.heads[r][i];
  if (hl.n == 0 || !p->rope) return VORTA_OK;
  const UserTensor ut = user_tensor(p, src);
  const int cs = chunk_shift(p);
  const long total = (long)p->N << cs;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  const Rope rope = make_rope(p);
  hipStream_t st = (hipStream_t)stream;
  if (p->d.dtype == VORTA_BF16)
    hipLaunchKernelGGL(rope_rows_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, (const uint16_t*)src, (uint16_t*)dst,
                       hl, (int)p->L, (int)p->N, ut.head_stride, ut.row_stride, cs, rope);
  else
    hipLaunchKernelGGL(rope_rows_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)src, (float*)dst, hl,
                       (int)p->L, (int)p->N, ut.head_stride, ut.row_stride, cs, rope);
  return launch_status("rope_rows_kernel");
}

// ------------------------------------------------------------------------------------------
// Router (Eq. 3) and hard selection (Eq. 4) for a whole sampling schedule: one wavefront per
// (step, head).  The gates depend on the timestep embedding only, so every step's routes can be
// had before sampling starts, in one launch.  The three logits are fp64 sums (lanes stride over
// d_t, then a fixed xor tree), the softmax is fp64, the gates are stored as fp32; Eq. 4 is
// decided on the fp64 gates, every tie going to full attention.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void router_kernel(const float* __restrict__ t_emb, const float* __restrict__ w_r,
                                                    int d_t, int heads, float* __restrict__ alpha,
                                                    uint8_t* __restrict__ routes) {
#pragma clang fp contract(off)
  const int h = blockIdx.x, step = blockIdx.y, lane = threadIdx.x;
  const float* t = t_emb + (long)step * d_t;
  const float* w = w_r + (long)h * d_t * 3;
  double z[3] = {0.0, 0.0, 0.0};
  for (int i = lane; i < d_t; i += 64) {
    const double ti = (double)t[i];
#pragma unroll
    for (int k = 0; k < 3; ++k) z[k] += ti * (double)w[3 * i + k];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1)
#pragma unroll
    for (int k = 0; k < 3; ++k) z[k] += __shfl_xor(z[k], off, 64);
  if (lane == 0) {
    const double m = fmax(z[0], fmax(z[1], z[2]));
    const double e0 = exp(z[0] - m), e1 = exp(z[1] - m), e2 = exp(z[2] - m);
    const double sum = e0 + e1 + e2;
    const double a1 = e0 / sum, a2 = e1 / sum, a3 = e2 / sum;
    float* out = alpha + ((long)step * heads + h) * 3;
    out[0] = (float)a1; out[1] = (float)a2; out[2] = (float)a3;
    uint8_t r = VORTA_ROUTE_FULL;
    if (a2 > a1 && a2 > a3) r = VORTA_ROUTE_WINDOW;
    else if (a3 > a1 && a3 > a2) r = VORTA_ROUTE_CORESET;
    routes[(long)step * heads + h] = r;
  }
}

int launch_router(const float* t_emb, const float* w_r, int n_steps, int d_t, int heads, float* alpha,
                  uint8_t* routes, void* stream) {
  hipLaunchKernelGGL(router_kernel, dim3(heads, n_steps), dim3(64), 0, (hipStream_t)stream, t_emb, w_r, d_t, heads,
                     alpha, routes);
  return launch_status("router_kernel");
}

// ------------------------------------------------------------------------------------------
// Eq. 5 blend: out = a1 o_full + a2 o_sliding + a3 o_coreset, gates per head
// ------------------------------------------------------------------------------------------
struct Gates {
  float a[VORTA_MAX_HEADS][3];
};

template <typename T>
__global__ __launch_bounds__(256) void blend_kernel(const T* __restrict__ o0, const T* __restrict__ o1,
                                                    const T* __restrict__ o2, T* __restrict__ out, Gates gt,
                                                    long total, int head_dim, int heads, long N, int layout) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const long row = i / head_dim;
  const int h = layout == VORTA_LAYOUT_NHD ? (int)(row % heads) : (int)(row / N);
  const double v = (double)gt.a[h][0] * Elem<T>::load(o0 + i) + (double)gt.a[h][1] * Elem<T>::load(o1 + i) +
                   (double)gt.a[h][2] * Elem<T>::load(o2 + i);
  Elem<T>::store(out + i, v);
}

int launch_blend3(vorta_plan* p, const void* o0, const void* o1, const void* o2, const float* alpha_host,
                  void* out, void* stream) {
  Gates gt;
  std::memset(&gt, 0, sizeof(gt));
  for (int h = 0; h < p->d.heads; ++h)
    for (int r = 0; r < 3; ++r) gt.a[h][r] = alpha_host[3 * h + r];
  const long total = (long)p->d.heads * p->N * p->d.head_dim;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipStream_t st = (hipStream_t)stream;
  if (p->d.dtype == VORTA_BF16)
    hipLaunchKernelGGL(blend_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, (const uint16_t*)o0,
                       (const uint16_t*)o1, (const uint16_t*)o2, (uint16_t*)out, gt, total, p->d.head_dim,
                       p->d.heads, (long)p->N, p->d.layout);
  else
    hipLaunchKernelGGL(blend_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)o0, (const float*)o1,
                       (const float*)o2, (float*)out, gt, total, p->d.head_dim, p->d.heads, (long)p->N,
                       p->d.layout);
  return launch_status("blend_kernel");
}

}  // namespace vorta
