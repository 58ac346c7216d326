// bf16 routed attention for gfx950 (CDNA4): flash-style forward.  Two kernels: a software-
// pipelined one (further down) that runs every segment of the layer call -- dense, core-set
// and, gathering rows through the tile permutation, the window tiles -- and a simpler one
// (first) for window tiles given as tile-ordered copies.  Common to both:
//
// A wavefront owns 32 query rows; keys stream through LDS in blocks of 64 rows.  Both contractions run on
// v_mfma_f32_32x32x16_bf16 and are computed TRANSPOSED so that a lane owns one query:
//     S^T = K Q^T      A = K rows from LDS (one ds_read_b128 per lane), B = Q^T kept in VGPRs
//     O^T += V^T P^T   A = V^T read from row-major V with ds_read_b64_tr_b16, B = P^T
// In the 32x32 accumulator layout lane l holds column (l & 31) = one query, so the row
// max / sum of the online softmax are in-lane reductions plus one exchange with lane l^32,
// the rescale of O^T is a per-lane scalar multiply, and exp(S) converted to bf16 is already
// in B-operand order: P never leaves registers.  (The k index of the second product is a
// permutation of the key index; V^T is read with the same permutation.)
// Softmax statistics are fp32, exp via v_exp_f32 on scores pre-multiplied by log2(e).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "vorta_attn_common.h"

namespace vorta {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

namespace {
constexpr int D = 128;          // head dim
constexpr int BM = 128;         // query rows per workgroup, window segment (4 wavefronts)
constexpr int BM_LONG = 256;    // dense and core-set segments (8 wavefronts)
constexpr int BN = 64;          // keys per LDS block
// LDS row strides in elements (256 B of data + pad), chosen per access pattern with the LDS
// bank-conflict counter: ds_read_b128 of 32 consecutive rows is conflict free at 272 B; the
// ds_read_b64_tr_b16 pattern (per instruction 8 rows x 64 B) needs its rows 64 B apart modulo
// 256 B, i.e. 320 B (at 288 B every such read takes twice the LDS cycles).
constexpr int LSTR = 136;       // K block and output staging
constexpr int VSTR = 160;       // V block
constexpr int KTILE64 = BN * LSTR;
constexpr int STAGE64_ELEMS = BN * (LSTR + VSTR);   // one K block + one V block
constexpr int LDS_BYTES = 2 * STAGE64_ELEMS * 2;
constexpr float P_MAX = 256.f;  // largest probability (relative to the row reference) the softmax fast path accepts
}  // namespace

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(unsigned, b);
}

__device__ __forceinline__ bf16x8 read_vt(const uint16_t* p_lo, const uint16_t* p_hi) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p_lo);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p_hi);
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

__device__ __forceinline__ float max3(float a, float b, float c) {
  return __builtin_fmaxf(__builtin_fmaxf(a, b), c);   // one v_max3_f32
}

// max of x over the lane pair (l, l ^ 32).  v_permlane32_swap exchanges the upper half of its
// first operand with the lower half of its second inside the vector ALU (no LDS round trip);
// the wait states around it are the ones the instruction needs after / before vector ALU
// accesses to the same registers.
__device__ __forceinline__ float max_xor32(float x) {
  float lo = x, hi = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(lo), "+v"(hi));
  return __builtin_fmaxf(lo, hi);
}

__device__ __forceinline__ bf16x8 lds_frag(const uint16_t* p) {
  return __builtin_bit_cast(bf16x8, *(const uint4*)p);
}

// LDS-address-space pointer flavours: a 32-bit base register plus immediate offsets.
typedef __attribute__((address_space(3))) const uint16_t* lds_ptr;
typedef __attribute__((address_space(3))) const uint4* lds_u4_ptr;
__device__ __forceinline__ bf16x8 lds_frag3(lds_ptr p) { return __builtin_bit_cast(bf16x8, *(lds_u4_ptr)p); }
__device__ __forceinline__ bf16x8 read_vt3(lds_ptr p_lo, lds_ptr p_hi) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p_lo);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p_hi);
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}
// Hide how a per-sub-step LDS base was computed, so every fragment read is base + immediate
// instead of one precomputed address register per fragment.
__device__ __forceinline__ lds_ptr opaque(lds_ptr p) {
  asm volatile("" : "+v"(p));
  return p;
}

typedef int i32x4 __attribute__((ext_vector_type(4)));

#define MFMA(a_, b_, c_) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, b_, c_, 0, 0, 0)

// Run list of a work item.  It is the same for every lane and no kernel writes it, so it is
// read as constant memory: with a wave-uniform index that is a scalar load, whose result lands
// in a scalar register and whose wait does not include the vector loads in flight.
typedef const __attribute__((address_space(4))) int* const_int_ptr;
struct RunList {
  const_int_ptr runs;      // (start, length) pairs; null: the single run {0, single_len}
  int n_runs, single_len;
  __device__ __forceinline__ explicit RunList(const WorkItem& w)
      : runs((const_int_ptr)(uintptr_t)w.runs), n_runs(w.n_runs), single_len(w.single_len) {}
  __device__ __forceinline__ int start(int r) const { return runs ? runs[2 * r] : 0; }
  __device__ __forceinline__ int len(int r) const { return runs ? runs[2 * r + 1] : single_len; }
};

// Rows of keys j0 + step i (i < NR) of the bn-key block that begins pos keys into run r, whose
// first row is s and whose length is len (r, pos, s, len wave-uniform; j0 per lane).  A block
// that reaches past the end of run r continues in the following runs: they are walked with
// uniform control flow, each lane keeping the row of the run its key falls in.  Keys past the
// end of the last run repeat its last row (they are masked out of the softmax).
template <int NR>
__device__ __forceinline__ void block_rows(const RunList& rl, int r, int pos, int s, int len, int bn, int j0, int step,
                                           int (&rows)[NR]) {
  int k[NR];
#pragma unroll
  for (int i = 0; i < NR; ++i) {
    k[i] = pos + j0 + step * i;
    rows[i] = s + min(k[i], len - 1);
  }
  int end = pos + bn;
  while (end > len && r + 1 < rl.n_runs) {
    end -= len;
#pragma unroll
    for (int i = 0; i < NR; ++i) k[i] -= len;
    ++r;
    s = rl.start(r);
    len = rl.len(r);
#pragma unroll
    for (int i = 0; i < NR; ++i)
      if (k[i] >= 0) rows[i] = s + min(k[i], len - 1);
  }
}


// Window segment over tile-ordered copies of Q, K, V (the staged call with q_t, k_t, v_t, o_t
// given): a tile's key set is a short list of runs of consecutive rows.
template <int NW>   // NW wavefronts per workgroup: 4 (two workgroups per CU)
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_bf16_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int STG_ROWS = 4 * NW, STG_PASSES = BN / STG_ROWS;   // staging: rows per pass, passes per block
  const WorkItem w = decode_item<32 * NW, D>(a, xcd_item(blockIdx.x, gridDim.x, NW == 4));
  const uint16_t* Q = (const uint16_t*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const uint16_t* K = (const uint16_t*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const uint16_t* V = (const uint16_t*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  uint16_t* O = (uint16_t*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  const unsigned row_stride = (unsigned)w.row_stride;   // rows * stride < 2^31 elements (checked on the host)
  if (w.n_rows <= 0) return;       // q-block past the end of a clipped tile

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;

  // Q^T fragments: lane = query (l32), 8 consecutive dims per 16-wide k slice
  bf16x8 qf[8];
  {
    const unsigned qrow = w.row(min(32 * wave + l32, w.n_rows - 1));
    const uint16_t* qp = Q + qrow * row_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * ks));
  }

  // global -> LDS staging: thread moves the 16-byte chunk (tid & 15) of rows (tid >> 4) + STG_ROWS i.
  // The key rows of an item are the concatenation of its runs, cut into blocks of BN: a block
  // that lies inside one run is addressed as (wave-uniform base of its first row) + (per-thread
  // byte offset that never changes), so its loads need no per-block vector address arithmetic;
  // a block that crosses into the next run(s) looks every row up in the run list, and the rows
  // past the end of the last run repeat its last row (they are masked out of the softmax).
  const int ld_row = tid >> 4, ld_col = (tid & 15) * 8;
  const unsigned ld_off0 = 2u * ((unsigned)ld_row * row_stride + (unsigned)ld_col);   // bytes
  const unsigned ld_step = 2u * STG_ROWS * row_stride;
  uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
#define FETCH_FULL(i_, kr_, vr_, kb_, vb_)                          \
  kr_ = *(const uint4*)((kb_) + (ld_off0 + (i_)*ld_step));           \
  vr_ = *(const uint4*)((vb_) + (ld_off0 + (i_)*ld_step));
#define FETCH_TAIL(kr_, vr_, row_)                                                         \
  {                                                                                        \
    const unsigned off_ = (unsigned)(row_) * row_stride + ld_col;                          \
    kr_ = *(const uint4*)(K + off_);                                                       \
    vr_ = *(const uint4*)(V + off_);                                                       \
  }
#define FETCH(run_, start_, len_, pos_)                                                    \
  if ((pos_) + BN <= (len_)) {                                                             \
    const size_t base_ = (size_t)(unsigned)((start_) + (pos_)) * row_stride * 2u;          \
    const char* kb_ = (const char*)K + base_;                                              \
    const char* vb_ = (const char*)V + base_;                                              \
    FETCH_FULL(0, kr0, vr0, kb_, vb_)                                                      \
    FETCH_FULL(1, kr1, vr1, kb_, vb_)                                                      \
    if constexpr (STG_PASSES == 4) {                                                       \
      FETCH_FULL(2, kr2, vr2, kb_, vb_)                                                    \
      FETCH_FULL(3, kr3, vr3, kb_, vb_)                                                    \
    }                                                                                      \
  } else {                                                                                 \
    int rows_[STG_PASSES];                                                                 \
    block_rows<STG_PASSES>(rl, run_, pos_, start_, len_, BN, ld_row, STG_ROWS, rows_);         \
    FETCH_TAIL(kr0, vr0, rows_[0])                                                         \
    FETCH_TAIL(kr1, vr1, rows_[1])                                                         \
    if constexpr (STG_PASSES == 4) {                                                       \
      FETCH_TAIL(kr2, vr2, rows_[2])                                                       \
      FETCH_TAIL(kr3, vr3, rows_[3])                                                       \
    }                                                                                      \
  }
#define STAGE(buf_)                                                       \
  {                                                                       \
    uint16_t* kb_ = smem + (buf_)*STAGE64_ELEMS + ld_row * LSTR + ld_col;   \
    uint16_t* vb_ = smem + (buf_)*STAGE64_ELEMS + KTILE64 + ld_row * VSTR + ld_col; \
    *(uint4*)(kb_) = kr0;                                                 \
    *(uint4*)(kb_ + STG_ROWS * LSTR) = kr1;                               \
    *(uint4*)(vb_) = vr0;                                                 \
    *(uint4*)(vb_ + STG_ROWS * VSTR) = vr1;                               \
    if constexpr (STG_PASSES == 4) {                                      \
      *(uint4*)(kb_ + 2 * STG_ROWS * LSTR) = kr2;                         \
      *(uint4*)(kb_ + 3 * STG_ROWS * LSTR) = kr3;                         \
      *(uint4*)(vb_ + 2 * STG_ROWS * VSTR) = vr2;                         \
      *(uint4*)(vb_ + 3 * STG_ROWS * VSTR) = vr3;                         \
    }                                                                     \
  }
  const RunList rl(w);
  auto run_start = [&](int r) { return rl.start(r); };
  auto run_len = [&](int r) { return rl.len(r); };

  int n_keys = 0;
  for (int r = 0; r < w.n_runs; ++r) n_keys += run_len(r);
  const int n_blocks = (n_keys + BN - 1) / BN;

  f32x16 o0, o1, o2, o3;
#pragma unroll
  for (int v = 0; v < 16; ++v) { o0[v] = 0.f; o1[v] = 0.f; o2[v] = 0.f; o3[v] = 0.f; }
  float m_run = -INFINITY, l_run = 0.f;
  const float c = a.scale * 1.4426950408889634f;

  // fetch cursor (run, offset in it, its first row and length): the next block to request
  int fr = 0, fpos = 0, fstart = run_start(0), flen = run_len(0), left = n_keys;
  auto advance = [&]() {
    fpos += BN;
    while (fpos >= flen && fr + 1 < w.n_runs) {
      fpos -= flen;
      ++fr;
      fstart = run_start(fr);
      flen = run_len(fr);
    }
  };
  // Prologue: block 0 goes to LDS, the rows of block 1 wait in the staging registers.  Iteration
  // it then writes block it + 1 to the other buffer first thing and requests block it + 2, so
  // a row has a whole iteration to arrive.
  FETCH(fr, fstart, flen, fpos)
  advance();
  STAGE(0)
  if (n_blocks > 1) {
    FETCH(fr, fstart, flen, fpos)
    advance();
  }
  __syncthreads();

  // per-lane LDS read offsets
  const uint16_t* k_rd = smem + l32 * LSTR + 8 * g;
  const int t16 = lane & 15, blk = lane >> 4;
  const uint16_t* v_rd = smem + KTILE64 + (4 * g + (t16 >> 2)) * VSTR + 16 * (blk & 1) + 4 * (t16 & 3);

  for (int it = 0; it < n_blocks; ++it) {
    if (it + 1 < n_blocks) { STAGE((it + 1) & 1) }        // rows requested an iteration ago
    if (it + 2 < n_blocks) {
      FETCH(fr, fstart, flen, fpos)
      advance();
    }

    const int n_valid = min(BN, left);
    const uint16_t* kp = k_rd + (it & 1) * STAGE64_ELEMS;
    const uint16_t* vp = v_rd + (it & 1) * STAGE64_ELEMS;

    // ---- S^T = K Q^T for keys [0,32) and [32,64) of the block
    f32x16 s0, s1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { s0[v] = 0.f; s1[v] = 0.f; }
    {
      bf16x8 f0 = lds_frag(kp), f1 = lds_frag(kp + 32 * LSTR);
      bf16x8 f2 = lds_frag(kp + 16), f3 = lds_frag(kp + 32 * LSTR + 16);
      bf16x8 f4 = lds_frag(kp + 32), f5 = lds_frag(kp + 32 * LSTR + 32);
      bf16x8 f6 = lds_frag(kp + 48), f7 = lds_frag(kp + 32 * LSTR + 48);
      s0 = MFMA(f0, qf[0], s0); s1 = MFMA(f1, qf[0], s1);
      f0 = lds_frag(kp + 64); f1 = lds_frag(kp + 32 * LSTR + 64);
      s0 = MFMA(f2, qf[1], s0); s1 = MFMA(f3, qf[1], s1);
      f2 = lds_frag(kp + 80); f3 = lds_frag(kp + 32 * LSTR + 80);
      s0 = MFMA(f4, qf[2], s0); s1 = MFMA(f5, qf[2], s1);
      f4 = lds_frag(kp + 96); f5 = lds_frag(kp + 32 * LSTR + 96);
      s0 = MFMA(f6, qf[3], s0); s1 = MFMA(f7, qf[3], s1);
      f6 = lds_frag(kp + 112); f7 = lds_frag(kp + 32 * LSTR + 112);
      s0 = MFMA(f0, qf[4], s0); s1 = MFMA(f1, qf[4], s1);
      s0 = MFMA(f2, qf[5], s0); s1 = MFMA(f3, qf[5], s1);
      s0 = MFMA(f4, qf[6], s0); s1 = MFMA(f5, qf[6], s1);
      s0 = MFMA(f6, qf[7], s0); s1 = MFMA(f7, qf[7], s1);
      // keep the fragment reads ahead of their use: 8 reads in flight, then 2 per MFMA pair
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
    if (n_valid < BN) {   // run tail: element v of a tile is key 8 (v >> 2) + 4 g + (v & 3)
      const int nv0 = n_valid - 4 * g, nv1 = nv0 - 32;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (8 * (v >> 2) + (v & 3) >= nv0) s0[v] = -INFINITY;
        if (8 * (v >> 2) + (v & 3) >= nv1) s1[v] = -INFINITY;
      }
    }

    // ---- softmax against a lagging row reference m_run (this lane's query, its 32 keys; the
    // other 32 are in lane ^ 32).  The probabilities go straight to bf16 pairs in B-operand
    // order: k slice kk covers keys [16 kk, 16 kk + 16).  The row sums are plain fp32 adds of
    // the probabilities (not v_dot2c_f32_bf16 on the packed pairs: see the pipelined kernel).
    const float mc = m_run * c;
    unsigned u0[8], u1[8];
    float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float a0 = __builtin_amdgcn_exp2f(fmaf(s0[2 * j], c, -mc)), a1 = __builtin_amdgcn_exp2f(fmaf(s0[2 * j + 1], c, -mc));
      const float b0 = __builtin_amdgcn_exp2f(fmaf(s1[2 * j], c, -mc)), b1 = __builtin_amdgcn_exp2f(fmaf(s1[2 * j + 1], c, -mc));
      u0[j] = pack_bf16(a0, a1);
      u1[j] = pack_bf16(b0, b1);
      ps0 += a0 + a1;
      ps1 += b0 + b1;
    }
    float ps = ps0 + ps1;
    // Reference check: no probability exceeds its row sum, so ps <= P_MAX proves that no score
    // of the block was more than log2(P_MAX) above the reference.  Otherwise (always for the
    // first block, whose reference is -inf; afterwards only when a row maximum jumps) the block
    // is redone against the true running maximum: new reference, accumulators and sum rescaled
    // to it, probabilities recomputed from the scores.
    if (__any(!(ps <= P_MAX))) {
      float mx = max3(s0[0], s1[0], s0[1]);
#pragma unroll
      for (int v = 1; v < 15; ++v) mx = max3(mx, s1[v], s0[v + 1]);
      mx = max_xor32(fmaxf(mx, s1[15]));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);   // 0 for the first block
      m_run = m_new;
      const float mc2 = m_new * c;
      ps = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float a0 = __builtin_amdgcn_exp2f(fmaf(s0[2 * j], c, -mc2)), a1 = __builtin_amdgcn_exp2f(fmaf(s0[2 * j + 1], c, -mc2));
        const float b0 = __builtin_amdgcn_exp2f(fmaf(s1[2 * j], c, -mc2)), b1 = __builtin_amdgcn_exp2f(fmaf(s1[2 * j + 1], c, -mc2));
        u0[j] = pack_bf16(a0, a1);
        u1[j] = pack_bf16(b0, b1);
        ps += (a0 + a1) + (b0 + b1);
      }
      l_run *= alpha;
#pragma unroll
      for (int v = 0; v < 16; ++v) { o0[v] *= alpha; o1[v] *= alpha; o2[v] *= alpha; o3[v] *= alpha; }
    }
    l_run += ps;
    bf16x8 pf[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      pf[h] = __builtin_bit_cast(bf16x8, make_uint4(u0[4 * h], u0[4 * h + 1], u0[4 * h + 2], u0[4 * h + 3]));
      pf[2 + h] = __builtin_bit_cast(bf16x8, make_uint4(u1[4 * h], u1[4 * h + 1], u1[4 * h + 2], u1[4 * h + 3]));
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const uint16_t* vk = vp + 16 * kk * VSTR;
      const bf16x8 t0 = read_vt(vk, vk + 8 * VSTR);
      const bf16x8 t1 = read_vt(vk + 32, vk + 8 * VSTR + 32);
      const bf16x8 t2 = read_vt(vk + 64, vk + 8 * VSTR + 64);
      const bf16x8 t3 = read_vt(vk + 96, vk + 8 * VSTR + 96);
      o0 = MFMA(t0, pf[kk], o0);
      o1 = MFMA(t1, pf[kk], o1);
      o2 = MFMA(t2, pf[kk], o2);
      o3 = MFMA(t3, pf[kk], o3);
    }

    __syncthreads();
    left -= BN;
  }

  // ---- epilogue: normalise, transpose through LDS, store whole rows
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  uint16_t* st = smem + wave * 32 * LSTR;
#define STORE_TILE(dt_, acc_)                                                        \
  _Pragma("unroll") for (int q4 = 0; q4 < 4; ++q4) {                                 \
    uint2 u;                                                                         \
    u.x = pack_bf16(acc_[4 * q4] * inv, acc_[4 * q4 + 1] * inv);                     \
    u.y = pack_bf16(acc_[4 * q4 + 2] * inv, acc_[4 * q4 + 3] * inv);                 \
    *(uint2*)(st + l32 * LSTR + 32 * (dt_) + 8 * q4 + 4 * g) = u;                    \
  }
  STORE_TILE(0, o0) STORE_TILE(1, o1) STORE_TILE(2, o2) STORE_TILE(3, o3)
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (lane >> 4) + 4 * i;
    if (32 * wave + row < w.n_rows)
      *(uint4*)(O + (unsigned)w.row(32 * wave + row) * row_stride + (lane & 15) * 8) =
          *(const uint4*)(st + row * LSTR + (lane & 15) * 8);
  }
}


// ------------------------------------------------------------------------------------------
// Software-pipelined kernel (described for its main form: 8 wavefronts, 256 query rows, 64-key
// blocks, one workgroup per CU).  Every matrix instruction gets independent vector work to run
// in its shadow, inside the same wavefront:
//
//   iteration i:   matrix pipe   O^T += V^T(i-1) P^T(i-1)   then   S^T(i+1) = K(i+1) Q^T
//                  vector pipe   online softmax of S^T(i) -> P^T(i)   (independent of both)
//                  memory        block i+3: global -> LDS
//
// The iteration is written as 32 slots, one matrix instruction each, separated by scheduling
// fences: a slot also requests the LDS fragments of the matrix instruction LEAD slots later
// and carries a few instructions of the softmax (or of the staging).  The softmax keeps a
// lagging row reference instead of the running maximum (see the reference check in the loop
// body), so the accumulators O^T are rescaled only on a rarely taken branch at the END of
// iteration i, after P(i-1) V(i-1) went in and before P(i) V(i) does.  Score tiles and
// probability fragments alternate between two register sets from one iteration to the next, so
// nothing is copied.  One barrier per iteration.
//
// Staging: K and V rows go from global memory straight into LDS with buffer_load_dwordx4 ... lds
// -- no staging registers, no LDS write instructions.  Such a load writes the 64 lanes' 16-byte
// pieces to 1 KiB of consecutive LDS bytes starting at M0, while each lane's global address is
// free.  A stage therefore holds its rows in groups of four, one load per group, and the groups
// are padded apart so that fragment reads stay free of bank conflicts: 1040 B between K groups
// (ds_read_b128 wants the 16-byte pieces of 32 consecutive rows distinct modulo 512 B), 1088 B
// between V groups (the ds_read_b64_tr_b16 pattern wants consecutive rows 64 B apart).
//   64-key blocks: rows j, j+16, j+32, j+48 form group j, each row 256 consecutive bytes.
//   32-key blocks: rows j, j+8, j+16, j+24 form group j, and all four fall among the 32 rows one
//   ds_read_b128 covers, so the group is stored in 128-byte pieces: half h of the group's row q
//   at 512 h + 128 q.  (With 64-byte pieces at 256 c + 64 G every K read took twice its LDS
//   cycles, by the bank-conflict counter.)
// Wavefront w loads groups w and w + NWV of K and of V: four loads per iteration.  K blocks live
// in a ring of four stages, V blocks in a ring of five: in iteration i, V(i-1) and K(i+1) are
// read (and, at its end, the first fragments of V(i)), block i+2 is landing and block i+3 is
// requested.  The loads are inline assembly, invisible to the compiler's wait-count bookkeeping,
// which would otherwise drain them before every LDS read; the kernel waits itself: before the
// barrier of iteration i, vmcnt leaves only this iteration's loads outstanding, so block i+2 is
// in LDS -- two iterations of latency cover.
// ------------------------------------------------------------------------------------------
namespace {
constexpr int KG = 520, VG = 544;        // elements from one four-row group of a K / V stage to the next (1 KiB + pad)
constexpr int K_RING = 4, V_RING = 5;    // stages
constexpr int pipe_lds_bytes(int nwv) { return (K_RING * KG + V_RING * VG) * (2 * nwv) * 2; }   // 2 nwv groups per stage
constexpr int LEAD = 2;                  // slots between a fragment request and its use (2..6 measured alike; 2 needs the fewest registers)
}  // namespace

__device__ __forceinline__ float elem_of(const f32x16& t0, const f32x16& t1, int e) { return e < 16 ? t0[e] : t1[e - 16]; }

// WIN: window items read through the tile permutation: the item's rows are tile-order indices
// into the caller's tensors -- every query, key, value and output row goes through a.tok_of
// (tile-order index -> token index) instead of living in tile-ordered copies; the key rows are
// the concatenation of the tile's runs cut into blocks.  The token indices of a key block are
// looked up one block ahead of its rows, so the two dependent loads never wait for each other
// inside one iteration.
// NWV: wavefronts per workgroup.  8: 256 query rows, 64-key blocks, one workgroup per CU (dense,
// core-set, window tiles of more than 128 tokens).  4: 128 query rows, 32-key blocks, half the
// ring, two workgroups per CU (smaller window tiles): the iteration has 16 slots instead of 32.
// MIX: the launch is the last of the three branches of Eq. 5 (dense items over every head) and
// its epilogue writes the gate-weighted sum of the three (see MixArgs).
template <bool WIN, int NWV, bool MIX = false>
__global__ __launch_bounds__(64 * NWV, 8 / NWV) void attn_bf16_pipe_kernel(const AttnArgs a,
                                                                            const std::conditional_t<MIX, MixArgs, NoMix> mx) {
  static_assert(!(MIX && WIN), "the Eq. 5 epilogue belongs to the dense launch");
  static_assert(pipe_lds_bytes(NWV) <= 160 * 1024, "K and V rings exceed the 160 KB of LDS of a CU");
  static_assert(32 * NWV * LSTR * 2 <= pipe_lds_bytes(NWV), "output staging does not fit in the rings it reuses");
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int KB = 8 * NWV;               // keys per block: 64 (8 wavefronts) or 32 (4)
  constexpr int NS = KB / 2;                // slots = matrix instructions per iteration
  constexpr int NPV = NS / 2;               // of which second-product slots (then NS - NPV score slots)
  constexpr int NE = KB / 2;                // score elements per lane and block
  constexpr int NP = NE / 2;                // bf16 pairs of probabilities per lane and block
  constexpr int NKS = KB / 16;              // 16-key k slices of the second product
  static_assert(NWV == 8 || NWV == 4, "8 wavefronts x 64-key blocks or 4 wavefronts x 32-key blocks");
  constexpr int NG = KB / 4;                // four-row groups per stage: group j holds rows j, j + NG, j + 2 NG, j + 3 NG
  constexpr int K_STAGE = NG * KG, V_STAGE = NG * VG;   // elements of a K / V stage
  constexpr int V_BASE = K_RING * K_STAGE;  // the K ring, then the V ring
  auto vstage = [](int b) { return (int)((unsigned)b % (unsigned)V_RING); };   // ring stage of V block b (K: b & 3)
  const WorkItem w = decode_item<32 * NWV, D>(a, xcd_item(blockIdx.x, gridDim.x, WIN));
  const uint16_t* Q = (const uint16_t*)(w.seg == 0 || WIN ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const uint16_t* K = (const uint16_t*)(w.seg == 0 || WIN ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const uint16_t* V = (const uint16_t*)(w.seg == 0 || WIN ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  uint16_t* O = (uint16_t*)(w.seg == 0 || WIN ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  const unsigned row_stride = (unsigned)w.row_stride;

  if (w.n_rows <= 0) return;       // no rows: second half of a split item, or a q-block past the end of a clipped tile

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;

  bf16x8 qf[8];
  {
    unsigned qrow = w.row(min(32 * wave + l32, w.n_rows - 1));
    if (WIN) qrow = (unsigned)a.tok_of[qrow];
    const uint16_t* qp = Q + qrow * row_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * ks));
  }

  const RunList rl(w);
  auto run_start = [&](int r) { return rl.start(r); };
  auto run_len = [&](int r) { return rl.len(r); };
  int n_keys = 0;
  for (int r = 0; r < w.n_runs; ++r) n_keys += run_len(r);
  const int n_blocks = (n_keys + KB - 1) / KB;   // dense / core-set: one run

  // ---- staging: a lane moves one 16-byte chunk of two rows of the block, of K and of V: its
  // wavefront loads groups wave and wave + NWV, and lane p of a load fills bytes 16 p .. 16 p + 15
  // of the group -- which of the group's four rows (ld_q) and which chunk of that row follows
  // from the group layout.  The fetch stream walks the run list one block per call and stays on
  // the last block once it is past the end (those extra copies land in ring stages nobody
  // reads), so the loads need no guard.
  const int ld_q = KB == 64 ? lane >> 4 : (lane >> 3) & 3;
  const int ld_chunk = KB == 64 ? lane & 15 : 8 * (lane >> 5) + (lane & 7);
  const int ld_row = wave + NG * ld_q, ld_col = 8 * ld_chunk;
  constexpr int STG_STEP = NWV;    // rows from a lane's first staging row to its second
  int fr = 0, fpos = 0, fstart = run_start(0), flen = run_len(0);
  unsigned f_row0 = 0, f_lim = 0;
  auto fetch_cursor = [&]() {      // first row and last valid row offset of the block, then advance
    f_row0 = (unsigned)(fstart + fpos);
    f_lim = (unsigned)(flen - 1 - fpos);
    if (fpos + KB < flen) {
      fpos += KB;
    } else if (fr + 1 < w.n_runs) {
      ++fr;
      fpos = 0;
      fstart = run_start(fr);
      flen = run_len(fr);
    }
  };
  auto row_off = [&](int i) {      // element offset of this thread's chunk in staging row i
    return __umul24(f_row0 + min((unsigned)(ld_row + STG_STEP * i), f_lim), row_stride) + (unsigned)ld_col;
  };
  // K / V rows come through buffer loads: a scalar resource descriptor per tensor (raw buffer, no
  // range check: offsets are in bounds by construction) plus one 32-bit byte offset per lane.
  // The hardware reads the lane offset as unsigned, so the 2^31 elements a tensor may hold (the
  // plan's limit) are all within reach; both factors of the row product stay below 2^24.
  // The descriptor is four scalar words (base, base high bits with stride 0, no range check, raw
  // 32-bit data format); lane p's 16 bytes at element offset off land at lds_addr + 16 p.  M0
  // carries the LDS address (one wait state between its write and its use).
  const unsigned long long k_pa = (unsigned long long)K, v_pa = (unsigned long long)V;
  const i32x4 rs_k = {__builtin_amdgcn_readfirstlane((int)(unsigned)k_pa), __builtin_amdgcn_readfirstlane((int)((unsigned)(k_pa >> 32) & 0xffffu)), -1, 0x00020000};
  const i32x4 rs_v = {__builtin_amdgcn_readfirstlane((int)(unsigned)v_pa), __builtin_amdgcn_readfirstlane((int)((unsigned)(v_pa >> 32) & 0xffffu)), -1, 0x00020000};
  const unsigned lds0 = (unsigned)(uintptr_t)(lds_ptr)smem;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma16 = [&](const i32x4& rs, unsigned lds_addr, unsigned off) {
    asm volatile("s_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"{m0}"(lds_addr), "v"(off * 2u), "s"(rs) : "memory");
  };
  // group wave + NWV h of K / V block b (h = 0, 1: this lane's first and second staging row)
  auto dma_k = [&](int h, int b, unsigned off) { dma16(rs_k, lds0 + 2u * (unsigned)((b & 3) * K_STAGE + (wave_u + NWV * h) * KG), off); };
  auto dma_v = [&](int h, int b, unsigned off) { dma16(rs_v, lds0 + 2u * (unsigned)(V_BASE + vstage(b) * V_STAGE + (wave_u + NWV * h) * VG), off); };
  // WIN: token indices of this thread's two staging rows of the NEXT block whose rows will be
  // loaded (gi0, gi1), looked up one block ahead of the rows; win_at / win_idx produce them for
  // the block under the fetch cursor (uniform parameters first, then the per-lane lookup).
  int gi0 = 0, gi1 = 0;
  int wi_run = 0, wi_pos = 0, wi_start = 0, wi_len = 1;
  auto win_at = [&]() {            // note the block under the cursor, advance the cursor (scalar work only)
    wi_run = fr;
    wi_pos = fpos;
    wi_start = fstart;
    wi_len = flen;
    fpos += KB;
    while (fpos >= flen && fr + 1 < w.n_runs) {
      fpos -= flen;
      ++fr;
      fstart = run_start(fr);
      flen = run_len(fr);
    }
  };
  // The lookups are loads the compiler does not see either (it would wait for them with
  // vmcnt(0), which also drains the row loads requested after them): they are requested BEFORE
  // the row loads of their iteration, so that win_wait -- everything but the last four vector
  // memory operations complete -- returns as soon as the indices are there, whatever the row
  // loads behind them are doing (the counter retires in order).
  auto win_idx = [&]() {           // token indices of the noted block
    int rows[2];
    block_rows<2>(rl, wi_run, wi_pos, wi_start, wi_len, KB, ld_row, STG_STEP, rows);
    asm volatile("global_load_dword %0, %2, %4\n\tglobal_load_dword %1, %3, %4"
                 : "=&v"(gi0), "=&v"(gi1)
                 : "v"(rows[0] * 4), "v"(rows[1] * 4), "s"(a.tok_of)
                 : "memory");
  };
  auto win_wait = [&](bool rows_behind) {   // indices usable; rows_behind: four row loads were requested after them
    if (rows_behind) asm volatile("s_waitcnt vmcnt(4)" : "+v"(gi0), "+v"(gi1)::"memory");
    else asm volatile("s_waitcnt vmcnt(0)" : "+v"(gi0), "+v"(gi1)::"memory");
  };
  auto win_off = [&](int gi) { return __umul24((unsigned)gi, row_stride) + (unsigned)ld_col; };
  auto fetch_all = [&](int b, bool first = false) {   // rows of the block under the cursor, block b, into its ring stages
    unsigned o0_, o1_;
    if constexpr (WIN) {
      win_wait(!first);
      o0_ = win_off(gi0);
      o1_ = win_off(gi1);
      win_at();
      win_idx();                   // indices of the block after it
    } else {
      fetch_cursor();
      o0_ = row_off(0);
      o1_ = row_off(1);
    }
    dma_k(0, b, o0_); dma_v(0, b, o0_);
    dma_k(1, b, o1_); dma_v(1, b, o1_);
  };
  // valid keys of the blocks in compute order
  int cr = 0, cpos = 0, clen = flen, cblk = 0;
  auto next_valid = [&]() {      // 0 past the last block: a block of masked keys adds nothing
    if constexpr (WIN) {
      const int nv = min(KB, max(0, n_keys - KB * cblk));
      ++cblk;
      return nv;
    }
    const int nv = cblk < n_blocks ? min(KB, clen - cpos) : 0;
    ++cblk;
    if (cpos + KB < clen) {
      cpos += KB;
    } else if (cr + 1 < w.n_runs) {
      ++cr;
      cpos = 0;
      clen = run_len(cr);
    }
    return nv;
  };

  if constexpr (WIN) {             // prime the index pipeline with block 0
    win_at();
    win_idx();
  }
  fetch_all(0, true);              // blocks 0, 1 and 2 into their stages; iteration i requests block i+3
  fetch_all(1);
  fetch_all(2);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // Fragment addresses of the lane in stage 0 (elements), and what to add for further fragments.
  // 64-key blocks: row r sits in group r % 16 at (r / 16) * 256 B, chunks in order.
  // 32-key blocks: row r sits in group r % 8, half h of it at 512 h + 128 (r / 8) B.
  const int t16 = lane & 15, blk = lane >> 4;
  const lds_ptr k_rd = KB == 64 ? (lds_ptr)(smem + (l32 & 15) * KG + (l32 >> 4) * 128 + 8 * g)
                                : (lds_ptr)(smem + (l32 & 7) * KG + (l32 >> 3) * 64 + 8 * g);
  const lds_ptr v_rd = (lds_ptr)(smem + V_BASE + (4 * g + (t16 >> 2)) * VG + 16 * (blk & 1) + 4 * (t16 & 3));
  constexpr int K_T2 = 256;                                  // 64-key blocks: second 32-key tile
  auto k_slice = [](int ks) { return KB == 64 ? 16 * ks : 16 * (ks & 3) + 256 * (ks >> 2); };   // head-dim columns 16 ks ..
  auto v_cols = [](int cb) { return KB == 64 ? 32 * cb : 32 * (cb & 1) + 256 * (cb >> 1); };     // head-dim columns 32 cb ..
  constexpr int V_R16 = 128, V_R8 = KB == 64 ? 8 * VG : 64;  // 16 and 8 rows further

  f32x16 o[4], sa0, sa1, sb0, sb1;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    o[0][v] = 0.f; o[1][v] = 0.f; o[2][v] = 0.f; o[3][v] = 0.f;
    sa0[v] = 0.f; sa1[v] = 0.f; sb0[v] = 0.f; sb1[v] = 0.f;
  }
  float m_ref = -INFINITY, l_run = 0.f;   // row reference (a lagging running maximum) and row sum
  const float c = a.scale * 1.4426950408889634f;
  bf16x8 pa[NKS], pb[NKS];
#pragma unroll
  for (int i = 0; i < NKS; ++i) pa[i] = pb[i] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));

  // element v of a 32-key score tile is key 8 (v >> 2) + 4 g + (v & 3)
  auto mask_tail = [&](f32x16& t0, f32x16& t1, int n_valid) {
    const int nv0 = n_valid - 4 * g, nv1 = nv0 - 32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      if (8 * (v >> 2) + (v & 3) >= nv0) t0[v] = -INFINITY;
      if (KB == 64 && 8 * (v >> 2) + (v & 3) >= nv1) t1[v] = -INFINITY;
    }
  };

  // scores of block 0
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    sa0 = MFMA(lds_frag3(k_rd + k_slice(ks)), qf[ks], sa0);
    if constexpr (KB == 64) sa1 = MFMA(lds_frag3(k_rd + K_T2 + k_slice(ks)), qf[ks], sa1);
  }
  {
    const int nv = next_valid();
    if (nv < KB) mask_tail(sa0, sa1, nv);
  }

#define SLOT_FENCE() __builtin_amdgcn_sched_barrier(0)
  // first V^T fragments of the coming iteration, requested before the barrier of this one
  bf16x8 vpre[LEAD];
  auto v_frag = [&](lds_ptr vq, int n) {
    const lds_ptr ap = vq + V_R16 * (n >> 2) + v_cols(n & 3);
    return read_vt3(ap, ap + V_R8);
  };
#pragma unroll
  for (int n = 0; n < LEAD; ++n) vpre[n] = v_frag(v_rd, n);       // iteration 0 multiplies stage 0 by P = 0
  // One iteration.  sc*: scores of block i (in), sn*: scores of block i+1 (out),
  // pp: P^T(i-1) (in), pc: P^T(i) (out).
  auto body = [&](int i, f32x16& sc0, f32x16& sc1, f32x16& sn0, f32x16& sn1, bf16x8 (&pp)[NKS], bf16x8 (&pc)[NKS]) {
    const lds_ptr vq = opaque(v_rd + vstage(i ? i - 1 : 0) * V_STAGE);
    const lds_ptr kq = opaque(k_rd + ((i + 1) & 3) * K_STAGE);
    if constexpr (WIN) win_at();                     // block i+4: its token indices are looked up in slot 27
    else fetch_cursor();                             // block i+3 (scalar work and branches: before the slots)
    bf16x8 vf[NPV], kf[NS - NPV];
    auto v_req = [&](int n) { vf[n] = v_frag(vq, n); };
    auto k_req = [&](int n) { kf[n] = lds_frag3(KB == 64 ? kq + K_T2 * (n & 1) + k_slice(n >> 1) : kq + k_slice(n)); };
    const lds_ptr vq_next = opaque(v_rd + vstage(i) * V_STAGE);     // V(i): second product of iteration i+1
#pragma unroll
    for (int n = 0; n < LEAD; ++n) vf[n] = vpre[n];
    float ps0 = 0.f, ps1 = 0.f;
    float x[NE], ex[NE];
    unsigned u[2][8];                  // pair p of the block is u[p >> 3][p & 7]
    const float mc = m_ref * c;
    unsigned off0 = 0, off1 = 0;
#pragma unroll
    for (int n = 0; n < NS; ++n) {
      SLOT_FENCE();
      // ---- matrix instruction of the slot
      if (n < NPV) {
        o[n & 3] = MFMA(vf[n], pp[n >> 2], o[n & 3]);
      } else {
        const int m = n - NPV;
        if (m == 0) {
#pragma unroll
          for (int v = 0; v < 16; ++v) sn0[v] = 0.f;
        }
        if (KB == 64 && m == 1) {
#pragma unroll
          for (int v = 0; v < 16; ++v) sn1[v] = 0.f;
        }
        if constexpr (KB == 64) {      // two key tiles, alternating
          if (m & 1) sn1 = MFMA(kf[m], qf[m >> 1], sn1);
          else sn0 = MFMA(kf[m], qf[m >> 1], sn0);
        } else {
          sn0 = MFMA(kf[m], qf[m], sn0);
        }
      }
      // ---- fragment requests for the slot LEAD ahead
      if (n + LEAD < NPV) v_req(n + LEAD);
      else if (n + LEAD < NS) k_req(n + LEAD - NPV);
      else vpre[n + LEAD - NS] = v_frag(vq_next, n + LEAD - NS);
      // ---- vector work in the shadow of the matrix instruction: the probabilities of block i
      // relative to the row reference m_ref, spread evenly over the slots and staggered by
      // stage so that no instruction of a slot waits for another one of the same slot (a
      // wavefront issues in order): slot n scales element n+1, exponentiates element n-1, adds
      // element n-2 to the row sum and (odd n) packs pair (n-3)/2.  The row sum is a plain fp32
      // add per element: v_dot2c_f32_bf16 on the packed pairs would be half the instructions,
      // but it runs on the matrix pipe -- one per slot next to the matrix instruction costs
      // 45 % of the matrix rate in a register-only microbenchmark, two v_add_f32 cost 2 %.
      // Element e < 16 is sc0[e], element e >= 16 is sc1[e - 16]; pair p = elements 2p, 2p+1.
      auto elem = [&](int e) { return e < 16 ? sc0[e] : sc1[e - 16]; };
      if (n == 0) { x[0] = fmaf(elem(0), c, -mc); x[1] = fmaf(elem(1), c, -mc); }
      if (n >= 1 && n <= NS - 2) x[n + 1] = fmaf(elem(n + 1), c, -mc);
      if (n >= 1 && n <= NS - 2) ex[n - 1] = __builtin_amdgcn_exp2f(x[n - 1]);
      if (n == NS - 1) { ex[NE - 2] = __builtin_amdgcn_exp2f(x[NE - 2]); ex[NE - 1] = __builtin_amdgcn_exp2f(x[NE - 1]); }
      if (n >= 3 && (n & 1)) {
        const int p = (n - 3) >> 1;
        u[p >> 3][p & 7] = pack_bf16(ex[2 * p], ex[2 * p + 1]);
        asm volatile("" : "+v"(u[p >> 3][p & 7]));   // used next iteration: keep its computation in this slot
      }
      if (n >= 2) {
        if (n & 1) ps1 += ex[n - 2];
        else ps0 += ex[n - 2];
      }
      // ---- staging: the rows of block i+3 are requested -- addresses in slot SO, the four loads
      // from slot SL + 1 on, SP slots apart (32 slots: spread over the iteration; 16 slots: in
      // a row) -- and (WIN) the token indices of block i+4 looked up in slot SI, right after the
      // addresses, which were the last use of the indices they replace, and ahead of the row
      // loads, so that waiting for them a whole iteration later does not wait for those.
      constexpr int SL = NS == 32 ? 8 : 9, SP = NS == 32 ? 4 : 1;
      constexpr int SO = WIN ? 1 : SL, SI = 2;
      if (n == SO) {
        if constexpr (WIN) win_wait(true);
        off0 = WIN ? win_off(gi0) : row_off(0);
        off1 = WIN ? win_off(gi1) : row_off(1);
      }
      if (WIN && n == SI) win_idx();
      if (n == SL + 1) dma_k(0, i + 3, off0);
      if (n == SL + 1 + SP) dma_v(0, i + 3, off0);
      if (n == SL + 1 + 2 * SP) dma_k(1, i + 3, off1);
      if (n == SL + 1 + 3 * SP) dma_v(1, i + 3, off1);
    }
    SLOT_FENCE();
    constexpr int LP = NP - 1;         // last pair: packed here, its two elements summed
    u[LP >> 3][LP & 7] = pack_bf16(ex[NE - 2], ex[NE - 1]);
    ps0 += ex[NE - 2];
    ps1 += ex[NE - 1];
    float ps = ps0 + ps1;
    asm volatile("" : "+v"(u[LP >> 3][LP & 7]), "+v"(ps));
    // all but this iteration's memory operations (four row loads, WIN: and two index lookups) are
    // complete: the rows requested in the previous iteration are in LDS
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(WIN ? 6 : 4) : "memory");
    __syncthreads();
    // ---- reference check.  No probability exceeds its row sum, so ps <= P_MAX proves that no
    // score of the block was more than log2(P_MAX) above the reference.  Otherwise (always for
    // the first block, whose reference is -inf; afterwards only when a row maximum jumps) the
    // block is redone against the true running maximum: new reference, accumulators and sum
    // rescaled to it, probabilities recomputed from the scores, which are still in registers.
    if (__any(!(ps <= P_MAX))) {
      float mx;
      if constexpr (KB == 64) {
        mx = max3(sc0[0], sc1[0], sc0[1]);
#pragma unroll
        for (int k = 1; k < 15; ++k) mx = max3(mx, sc1[k], sc0[k + 1]);
        mx = fmaxf(mx, sc1[15]);
      } else {
        mx = max3(sc0[0], sc0[1], sc0[2]);
#pragma unroll
        for (int k = 3; k < 15; k += 2) mx = max3(mx, sc0[k], sc0[k + 1]);
        mx = fmaxf(mx, sc0[15]);
      }
      mx = max_xor32(mx);
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c);     // 0 for the first block
      m_ref = m_new;
      const float mc2 = m_new * c;
      ps = 0.f;
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const float e0 = __builtin_amdgcn_exp2f(fmaf(elem_of(sc0, sc1, 2 * p), c, -mc2));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(elem_of(sc0, sc1, 2 * p + 1), c, -mc2));
        u[p >> 3][p & 7] = pack_bf16(e0, e1);
        ps += e0 + e1;
      }
      l_run *= alpha;
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[d][v] *= alpha;
    }
    l_run += ps;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      pc[h] = __builtin_bit_cast(bf16x8, make_uint4(u[0][4 * h], u[0][4 * h + 1], u[0][4 * h + 2], u[0][4 * h + 3]));
      if constexpr (KB == 64)
        pc[2 + h] = __builtin_bit_cast(bf16x8, make_uint4(u[1][4 * h], u[1][4 * h + 1], u[1][4 * h + 2], u[1][4 * h + 3]));
    }
    const int nv = next_valid();
    if (nv < KB) mask_tail(sn0, sn1, nv);
  };
  // An even number of iterations, so the two register sets swap back; when the block count
  // is odd the last iteration works on a block of masked keys (probabilities 0) and only its
  // second product, of the real last block, matters.  The scores an iteration computes for
  // the block after the last one come from a ring stage holding a copy of the last block.
  if (32 * wave < w.n_rows) {
    for (int i = 0; i < n_blocks; i += 2) {
      body(i, sa0, sa1, sb0, sb1, pa, pb);
      body(i + 1, sb0, sb1, sa0, sa1, pb, pa);
    }
  } else {
    // helper wavefront (no query rows: upper half of a split item, or past the last row): it only
    // keeps its share of the staging going, with the same barriers as the others
    for (int i = 0; i < ((n_blocks + 1) & ~1); ++i) {
      fetch_all(i + 3);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(WIN ? 6 : 4) : "memory");
      __syncthreads();
    }
  }
#undef SLOT_FENCE

  // ---- second product of the last iteration's block (its probabilities are in pa)
  {
    const int last = ((n_blocks + 1) & ~1) - 1;
    const lds_ptr vq = opaque(v_rd + vstage(last) * V_STAGE);
#pragma unroll
    for (int n = 0; n < NPV; ++n)
      o[n & 3] = MFMA(n < LEAD ? vpre[n] : v_frag(vq, n), pa[n >> 2], o[n & 3]);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no row load is still on its way into the ring
  __syncthreads();   // every wavefront is done with the ring before stage 0 is reused below

  // ---- epilogue: normalise, transpose through LDS, store whole rows
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  uint16_t* st = smem + wave * 32 * LSTR;
  unsigned orow[8];                // looked up together, ahead of the barrier
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    orow[i] = w.row(min(32 * wave + (lane >> 4) + 4 * i, w.n_rows - 1));
    if (WIN) orow[i] = (unsigned)a.tok_of[orow[i]];
  }
  STORE_TILE(0, o[0]) STORE_TILE(1, o[1]) STORE_TILE(2, o[2]) STORE_TILE(3, o[3])
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (lane >> 4) + 4 * i;
    if (32 * wave + row < w.n_rows) {
      uint4 mine = *(const uint4*)(st + row * LSTR + (lane & 15) * 8);
      uint4* dst = (uint4*)(O + orow[i] * row_stride + (lane & 15) * 8);
      if constexpr (MIX) {
        const int tok = (int)orow[i];
        const bool video = tok < a.L;
        const int slot = video ? mx.assign[(long)w.head * a.L + tok] : mx.Lc + (tok - a.L);
        const uint4 core = *(const uint4*)((const uint16_t*)mx.oc + ((long)w.head * a.Nc + slot) * D + (lane & 15) * 8);
        const uint4 slide = video ? *dst : mine;
        const float a1 = mx.alpha[w.head][0], a2 = mx.alpha[w.head][1], a3 = mx.alpha[w.head][2];
        const unsigned f[4] = {mine.x, mine.y, mine.z, mine.w}, s2[4] = {slide.x, slide.y, slide.z, slide.w},
                       c3[4] = {core.x, core.y, core.z, core.w};
        unsigned r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = a1 * __uint_as_float(f[e] << 16) + a2 * __uint_as_float(s2[e] << 16) + a3 * __uint_as_float(c3[e] << 16);
          const float hi = a1 * __uint_as_float(f[e] & 0xffff0000u) + a2 * __uint_as_float(s2[e] & 0xffff0000u) +
                           a3 * __uint_as_float(c3[e] & 0xffff0000u);
          r[e] = pack_bf16(lo, hi);
        }
        mine = make_uint4(r[0], r[1], r[2], r[3]);
      }
      *dst = mine;
    }
  }
}

static int set_lds_limit(const void* kernel, const char* name, int bytes) {
  hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return fail(VORTA_EHIP, "hipFuncSetAttribute(%s, %d B LDS): %s", name, bytes, hipGetErrorString(e));
  return VORTA_OK;
}

// mix: the launch is the full-attention branch of Eq. 5 over the heads of route 0 and blends the
// other two branches in (their results must be complete on the stream).  win_text = false leaves
// out the text rows of the window heads (under Eq. 5 they equal the full-attention branch's).
int launch_attention_bf16(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream,
                          const MixArgs* mix, bool win_text) {
  static std::once_flag once;
  static int attr_rc = VORTA_OK;
  std::call_once(once, [] {
    attr_rc = set_lds_limit((const void*)attn_bf16_kernel<4>, "attn_bf16_kernel<4>", LDS_BYTES);
    if (!attr_rc) attr_rc = set_lds_limit((const void*)attn_bf16_pipe_kernel<false, 8>, "attn_bf16_pipe_kernel<false, 8>", pipe_lds_bytes(8));
    if (!attr_rc) attr_rc = set_lds_limit((const void*)attn_bf16_pipe_kernel<false, 8, true>, "attn_bf16_pipe_kernel<false, 8, true>", pipe_lds_bytes(8));
    if (!attr_rc) attr_rc = set_lds_limit((const void*)attn_bf16_pipe_kernel<true, 8>, "attn_bf16_pipe_kernel<true, 8>", pipe_lds_bytes(8));
    if (!attr_rc) attr_rc = set_lds_limit((const void*)attn_bf16_pipe_kernel<true, 4>, "attn_bf16_pipe_kernel<true, 4>", pipe_lds_bytes(4));
  });
  if (attr_rc) return attr_rc;
  if (mix && (rl.count[1] || rl.count[2])) return fail(VORTA_EINVAL, "the Eq. 5 epilogue takes full-attention heads only");
  // Long items -- dense heads, core-set heads and the text rows of the window heads, which
  // attend to every row -- run on the pipelined kernel in 256-row workgroups.
  RouteLists win_rl = rl;
  win_rl.count[0] = win_rl.count[2] = 0;
  AttnArgs a;
  if (int rc = fill_attn_args(p, rl, io, BM_LONG, win_text ? WIN_TEXT : WIN_NONE, &a)) return rc;
  if (a.end_tile > 0) {
    // the last items (at most one per two CUs) go out as half-row items: see AttnArgs::split_from
    const int n_split = std::min(a.end_tile, p->n_cus / 2);
    a.split_from = a.end_tile - n_split;
    if (mix)
      hipLaunchKernelGGL((attn_bf16_pipe_kernel<false, 8, true>), dim3(a.end_tile + n_split), dim3(512), pipe_lds_bytes(8), (hipStream_t)stream, a, *mix);
    else
      hipLaunchKernelGGL((attn_bf16_pipe_kernel<false, 8>), dim3(a.end_tile + n_split), dim3(512), pipe_lds_bytes(8), (hipStream_t)stream, a, NoMix());
  }
  // Window tiles.  Gathered from the caller's tensors (no tile-ordered copies given): the
  // pipelined kernel again -- tiles of more than 128 tokens in 256-row workgroups of 8
  // wavefronts, smaller tiles in 128-row workgroups of 4 wavefronts on 32-key blocks, two per CU.
  // Over tile-ordered copies: the plain 128-row kernel.
  const bool win_long = a.win_gather && p->tile_tokens > BM;
  const bool grouped = a.win_gather && !win_long && rl.count[1] > 0;
  if (grouped) {
    // tiles of at most 128 tokens, gathered: the plan's grouped items -- those of more than 128
    // rows (two or three tiles with one key set) on the 8-wavefront instance, the rest on the
    // 4-wavefront one
    if (int rc = fill_attn_args(p, win_rl, io, BM_LONG, WIN_TILES, &a, 0)) return rc;
    if (a.end_tile > 0) {
      const int n_split = std::min(a.end_tile, p->n_cus / 2);
      a.split_from = a.end_tile - n_split;
      hipLaunchKernelGGL((attn_bf16_pipe_kernel<true, 8>), dim3(a.end_tile + n_split), dim3(512), pipe_lds_bytes(8), (hipStream_t)stream, a, NoMix());
    }
    if (int rc = fill_attn_args(p, win_rl, io, BM, WIN_TILES, &a, 1)) return rc;
    if (a.end_tile > 0)
      hipLaunchKernelGGL((attn_bf16_pipe_kernel<true, 4>), dim3(a.end_tile), dim3(256), pipe_lds_bytes(4), (hipStream_t)stream, a, NoMix());
  } else {
    if (int rc = fill_attn_args(p, win_rl, io, win_long ? BM_LONG : BM, WIN_TILES, &a)) return rc;
    if (a.end_tile > 0 && win_long) {
      const int n_split = std::min(a.end_tile, p->n_cus / 2);
      a.split_from = a.end_tile - n_split;
      hipLaunchKernelGGL((attn_bf16_pipe_kernel<true, 8>), dim3(a.end_tile + n_split), dim3(512), pipe_lds_bytes(8), (hipStream_t)stream, a, NoMix());
    } else if (a.end_tile > 0) {
      hipLaunchKernelGGL((attn_bf16_kernel<4>), dim3(a.end_tile), dim3(256), LDS_BYTES, (hipStream_t)stream, a);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(VORTA_EHIP, "launch of attn_bf16 kernels: %s", hipGetErrorString(e));
  return VORTA_OK;
}

}  // namespace vorta

