// bf16 routed attention for gfx950 (CDNA4): flash-style forward, one launch for all heads.
//
// Workgroup = 4 wavefronts = 128 query rows (32 per wavefront); keys stream through LDS in
// blocks of 64 rows, double buffered, one barrier per block.  Both contractions run on
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

#include <cstdlib>
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
constexpr int BM = 128;         // query rows per workgroup
constexpr int BN = 64;          // keys per LDS block
// LDS row strides in elements (256 B of data + pad), chosen per access pattern from a
// bank-conflict microbenchmark: ds_read_b128 of 32 consecutive rows is conflict free at
// 272 B, the ds_read_b64_tr_b16 pattern (4 rows x 32 B per 16 lanes) at 288 B.
constexpr int LSTR = 136;       // K block and output staging
constexpr int VSTR = 144;       // V block
constexpr int KTILE = BN * LSTR;
constexpr int STAGE_ELEMS = BN * (LSTR + VSTR);   // one K block + one V block
constexpr int LDS_BYTES = 2 * STAGE_ELEMS * 2;
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
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
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

#define MFMA(a_, b_, c_) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, b_, c_, 0, 0, 0)

template <int NW>   // wavefronts per workgroup: 4 (two workgroups per CU) or 8 (one)
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_bf16_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int STG_ROWS = 4 * NW, STG_PASSES = BN / STG_ROWS;   // staging: rows per pass, passes per block
  const WorkItem w = decode_item<32 * NW, D>(a, blockIdx.x);
  const uint16_t* Q = (const uint16_t*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const uint16_t* K = (const uint16_t*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const uint16_t* V = (const uint16_t*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  uint16_t* O = (uint16_t*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  const unsigned row_stride = (unsigned)w.row_stride;   // rows * stride < 2^31 elements (checked on the host)

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;

  // Q^T fragments: lane = query (l32), 8 consecutive dims per 16-wide k slice
  bf16x8 qf[8];
  {
    const unsigned qrow = w.row0 + min(32 * wave + l32, w.n_rows - 1);
    const uint16_t* qp = Q + qrow * row_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * ks));
  }

  // global -> LDS staging: thread moves the 16-byte chunk (tid & 15) of rows (tid >> 4) + 16 i
  const int ld_row = tid >> 4, ld_col = (tid & 15) * 8;
  uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
#define FETCH_ROW(i_, kr_, vr_, start_, len_, pos_)                                        \
  {                                                                                        \
    const unsigned off_ = (unsigned)((start_) + min((pos_) + ld_row + STG_ROWS * (i_), (len_)-1)) * row_stride + ld_col; \
    kr_ = *(const uint4*)(K + off_);                                                       \
    vr_ = *(const uint4*)(V + off_);                                                       \
  }
#define FETCH(start_, len_, pos_)                      \
  FETCH_ROW(0, kr0, vr0, start_, len_, pos_)           \
  FETCH_ROW(1, kr1, vr1, start_, len_, pos_)           \
  if constexpr (STG_PASSES == 4) {                     \
    FETCH_ROW(2, kr2, vr2, start_, len_, pos_)         \
    FETCH_ROW(3, kr3, vr3, start_, len_, pos_)         \
  }
#define STAGE(buf_)                                                       \
  {                                                                       \
    uint16_t* kb_ = smem + (buf_)*STAGE_ELEMS + ld_row * LSTR + ld_col;   \
    uint16_t* vb_ = smem + (buf_)*STAGE_ELEMS + KTILE + ld_row * VSTR + ld_col; \
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
  auto run_start = [&](int r) { return w.runs ? w.runs[2 * r] : 0; };
  auto run_len = [&](int r) { return w.runs ? w.runs[2 * r + 1] : w.single_len; };

  int n_blocks = 0;
  for (int r = 0; r < w.n_runs; ++r) n_blocks += (run_len(r) + BN - 1) / BN;

  f32x16 o0, o1, o2, o3;
#pragma unroll
  for (int v = 0; v < 16; ++v) { o0[v] = 0.f; o1[v] = 0.f; o2[v] = 0.f; o3[v] = 0.f; }
  float m_run = -INFINITY, l_run = 0.f;
  const float c = a.scale * 1.4426950408889634f;

  int r = 0, pos = 0, start = run_start(0), len = run_len(0);
  FETCH(start, len, 0)
  STAGE(0)
  __syncthreads();

  // per-lane LDS read offsets
  const uint16_t* k_rd = smem + l32 * LSTR + 8 * g;
  const int t16 = lane & 15, blk = lane >> 4;
  const uint16_t* v_rd = smem + KTILE + (4 * g + (t16 >> 2)) * VSTR + 16 * (blk & 1) + 4 * (t16 & 3);

  for (int it = 0; it < n_blocks; ++it) {
    // cursor of the next block
    int nr = r, npos = pos + BN, nstart = start, nlen = len;
    if (npos >= len) {
      nr = r + 1;
      npos = 0;
      if (nr < w.n_runs) { nstart = run_start(nr); nlen = run_len(nr); }
    }
    const bool has_next = it + 1 < n_blocks;
    if (has_next) { FETCH(nstart, nlen, npos) }

    const int n_valid = min(BN, len - pos);
    const uint16_t* kp = k_rd + (it & 1) * STAGE_ELEMS;
    const uint16_t* vp = v_rd + (it & 1) * STAGE_ELEMS;

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
    }
    if (n_valid < BN) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 8 * (v >> 2) + 4 * g + (v & 3);
        if (key >= n_valid) s0[v] = -INFINITY;
        if (key + 32 >= n_valid) s1[v] = -INFINITY;
      }
    }

    // ---- online softmax: this lane's query, its 32 keys; the other 32 are in lane ^ 32
    float mx = max3(s0[0], s1[0], s0[1]);
    mx = max3(mx, s1[1], s0[2]);
#pragma unroll
    for (int v = 2; v < 15; ++v) mx = max3(mx, s1[v], s0[v + 1]);
    mx = fmaxf(mx, s1[15]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    if (__any(m_new > m_run)) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int v = 0; v < 16; ++v) { o0[v] *= alpha; o1[v] *= alpha; o2[v] *= alpha; o3[v] *= alpha; }
      m_run = m_new;
    }
    const float mc = m_run * c;
    float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s0[v] = __builtin_amdgcn_exp2f(fmaf(s0[v], c, -mc));
      s1[v] = __builtin_amdgcn_exp2f(fmaf(s1[v], c, -mc));
      ps0 += s0[v];
      ps1 += s1[v];
    }
    l_run += ps0 + ps1;

    // ---- P^T as B operands: k slice kk covers keys [16 kk, 16 kk + 16)
    bf16x8 pf[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint4 u0, u1;
      u0.x = pack_bf16(s0[8 * h + 0], s0[8 * h + 1]); u0.y = pack_bf16(s0[8 * h + 2], s0[8 * h + 3]);
      u0.z = pack_bf16(s0[8 * h + 4], s0[8 * h + 5]); u0.w = pack_bf16(s0[8 * h + 6], s0[8 * h + 7]);
      u1.x = pack_bf16(s1[8 * h + 0], s1[8 * h + 1]); u1.y = pack_bf16(s1[8 * h + 2], s1[8 * h + 3]);
      u1.z = pack_bf16(s1[8 * h + 4], s1[8 * h + 5]); u1.w = pack_bf16(s1[8 * h + 6], s1[8 * h + 7]);
      pf[h] = __builtin_bit_cast(bf16x8, u0);
      pf[2 + h] = __builtin_bit_cast(bf16x8, u1);
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

    if (has_next) { STAGE((it + 1) & 1) }
    __syncthreads();
    r = nr; pos = npos; start = nstart; len = nlen;
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
      *(uint4*)(O + (unsigned)(w.row0 + 32 * wave + row) * row_stride + (lane & 15) * 8) =
          *(const uint4*)(st + row * LSTR + (lane & 15) * 8);
  }
}

// ------------------------------------------------------------------------------------------
// Long-key-loop variant for the dense and core-set segments: 64 query rows per wavefront
// (two 32-row column blocks A and B), 256 rows per workgroup, one workgroup per CU.  Every K
// and V^T fragment read from LDS feeds two MFMAs, which halves the LDS traffic per FLOP -- the
// limiter of the 32-row kernel -- and the two blocks give the wavefront independent work to
// overlap softmax arithmetic with matrix instructions.
// ------------------------------------------------------------------------------------------
namespace {
constexpr int BM2 = 256;
}

// Softmax bookkeeping of the long-loop kernel ("lazy reference"): probabilities are taken
// relative to a per-query reference m_ref instead of the running maximum,
//     P' = exp2((s - m_ref) * scale * log2 e),   O' = sum P' V,   l' = sum P',   O = O' / l',
// which is the same quotient as long as nothing overflows.  The hot loop therefore never
// touches the O accumulators with vector ALU instructions.  When any score of a step exceeds
// m_ref by more than REF_SLACK (in log2 units, P' <= 2^REF_SLACK), the wavefront leaves the hot
// loop BEFORE using that step, raises m_ref to the running maximum, rescales O' and l' once,
// and re-enters the loop at the same step.  The first step always takes that path (m_ref
// starts at -inf).
constexpr float REF_SLACK = 8.0f;

__device__ __forceinline__ float max16(const f32x16& s) {
  float mx = max3(s[0], s[1], s[2]);
#pragma unroll
  for (int v = 3; v < 15; v += 2) mx = max3(mx, s[v], s[v + 1]);
  return fmaxf(mx, s[15]);
}

__device__ __forceinline__ void exp_pack(f32x16& s, float c, float mc, float& l, bf16x8& p0, bf16x8& p1) {
  float ps = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    s[v] = __builtin_amdgcn_exp2f(fmaf(s[v], c, -mc));
    ps += s[v];
  }
  l += ps;
  uint4 u0, u1;
  u0.x = pack_bf16(s[0], s[1]); u0.y = pack_bf16(s[2], s[3]); u0.z = pack_bf16(s[4], s[5]); u0.w = pack_bf16(s[6], s[7]);
  u1.x = pack_bf16(s[8], s[9]); u1.y = pack_bf16(s[10], s[11]); u1.z = pack_bf16(s[12], s[13]); u1.w = pack_bf16(s[14], s[15]);
  p0 = __builtin_bit_cast(bf16x8, u0);
  p1 = __builtin_bit_cast(bf16x8, u1);
}

__global__ __launch_bounds__(256, 1) void attn_bf16_m64_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int STG_ROWS = 16, STG_PASSES = 4;
  const WorkItem w = decode_item<BM2, D>(a, blockIdx.x);
  const uint16_t* Q = (const uint16_t*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const uint16_t* K = (const uint16_t*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const uint16_t* V = (const uint16_t*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  uint16_t* O = (uint16_t*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  const unsigned row_stride = (unsigned)w.row_stride;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;

  bf16x8 qa[8], qb[8];
  {
    const unsigned ra = w.row0 + min(64 * wave + l32, w.n_rows - 1);
    const unsigned rb = w.row0 + min(64 * wave + 32 + l32, w.n_rows - 1);
    const uint16_t* pa = Q + ra * row_stride + 8 * g;
    const uint16_t* pb = Q + rb * row_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qa[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(pa + 16 * ks));
      qb[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(pb + 16 * ks));
    }
  }

  const int ld_row = tid >> 4, ld_col = (tid & 15) * 8;
  uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
  auto run_start = [&](int r) { return w.runs ? w.runs[2 * r] : 0; };
  auto run_len = [&](int r) { return w.runs ? w.runs[2 * r + 1] : w.single_len; };
  int n_blocks = 0;
  for (int r = 0; r < w.n_runs; ++r) n_blocks += (run_len(r) + BN - 1) / BN;

  f32x16 a0, a1, a2, a3, b0, b1, b2, b3;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    a0[v] = 0.f; a1[v] = 0.f; a2[v] = 0.f; a3[v] = 0.f;
    b0[v] = 0.f; b1[v] = 0.f; b2[v] = 0.f; b3[v] = 0.f;
  }
  const float c = a.scale * 1.4426950408889634f;
  const float slack = REF_SLACK / c;                 // REF_SLACK in raw score units
  float mrefA = -INFINITY, mrefB = -INFINITY;        // per-query reference (same in lanes l, l^32)
  float mrunA = -INFINITY, mrunB = -INFINITY;        // this lane's running max (raw scores)
  float lA = 0.f, lB = 0.f;

  int r = 0, pos = 0, start = run_start(0), len = run_len(0);
  int nr = 0, npos = 0, nstart = 0, nlen = 0;
  FETCH(start, len, 0)
  STAGE(0)
  __syncthreads();

  const uint16_t* k_rd = smem + l32 * LSTR + 8 * g;
  const int t16 = lane & 15, blk = lane >> 4;
  const uint16_t* v_rd = smem + KTILE + (4 * g + (t16 >> 2)) * VSTR + 16 * (blk & 1) + 4 * (t16 & 3);

  const int n_steps = 2 * n_blocks;     // 32-key steps; two per LDS stage
  int j = 0;
  bool fetched = false;                 // next stage already requested (survives a re-entry)
  // FENCE pins the instruction order to the order written here -- a matrix instruction, then
  // a handful of vector instructions -- so a single wavefront keeps both pipes busy
  // (instructions issue in order).  PIN keeps speculative work on its side of a branch.
#define FENCE() __builtin_amdgcn_sched_barrier(0)
#define PIN(x_) asm volatile("" : "+v"(x_))
  while (j < n_steps) {
    bool raise = false;
    // -------- hot loop: no vector ALU instruction touches a*, b* in here --------
    // Step order: QK_A; QK_B with exp(A) in its shadow (speculative: uses the current reference
    // and is discarded if the check fails); reference check; PV_A with exp(B) in its shadow; PV_B.
    for (; j < n_steps; ++j) {
      const int it = j >> 1, h = j & 1;
      if (h == 0 && !fetched) {
        nr = r; npos = pos + BN; nstart = start; nlen = len;
        if (npos >= len) {
          nr = r + 1;
          npos = 0;
          if (nr < w.n_runs) { nstart = run_start(nr); nlen = run_len(nr); }
        }
        if (it + 1 < n_blocks) { FETCH(nstart, nlen, npos) }
        fetched = true;
      }
      // Keys past the end of a run are copies of its last row, so they never raise a row
      // maximum; only their probabilities have to be zeroed.
      const int n_valid = min(BN, len - pos) - 32 * h;     // valid keys of this step (may be <= 0)
      const uint16_t* kp = k_rd + (it & 1) * STAGE_ELEMS + 32 * h * LSTR;
      const uint16_t* vp = v_rd + (it & 1) * STAGE_ELEMS + 32 * h * VSTR;
      bf16x8 f[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) f[ks] = lds_frag(kp + 16 * ks);
      bf16x8 t[2][4];
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
          t[kk][dt] = read_vt(vp + 16 * kk * VSTR + 32 * dt, vp + (16 * kk + 8) * VSTR + 32 * dt);
      f32x16 sA, sB;
#pragma unroll
      for (int v = 0; v < 16; ++v) { sA[v] = 0.f; sB[v] = 0.f; }
      FENCE();
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) sA = MFMA(f[ks], qa[ks], sA);
      FENCE();
      const float mxA = max16(sA);
      const float mcA = mrefA * c, mcB = mrefB * c;
      float eA[16], eB[16];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        FENCE();
        sB = MFMA(f[i], qb[i], sB);
        FENCE();
        eA[2 * i] = __builtin_amdgcn_exp2f(fmaf(sA[2 * i], c, -mcA));
        eA[2 * i + 1] = __builtin_amdgcn_exp2f(fmaf(sA[2 * i + 1], c, -mcA));
        PIN(eA[2 * i]);
        PIN(eA[2 * i + 1]);
      }
      FENCE();
      const float mxB = max16(sB);
      mrunA = fmaxf(mrunA, mxA);
      mrunB = fmaxf(mrunB, mxB);
      if (__any(mxA > mrefA + slack || mxB > mrefB + slack)) {
        raise = true;
        break;                                            // step j is redone after the rescale
      }
      if (n_valid < 32) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (8 * (v >> 2) + 4 * g + (v & 3) >= n_valid) eA[v] = 0.f;
      }
      {
        float ps = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) ps += eA[v];
        lA += ps;
      }
      const bf16x8 pa0 = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(eA[0], eA[1]), pack_bf16(eA[2], eA[3]),
                                                                pack_bf16(eA[4], eA[5]), pack_bf16(eA[6], eA[7])));
      const bf16x8 pa1 = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(eA[8], eA[9]), pack_bf16(eA[10], eA[11]),
                                                                pack_bf16(eA[12], eA[13]), pack_bf16(eA[14], eA[15])));
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        FENCE();
        const bf16x8 pA = (i >> 2) ? pa1 : pa0;
        switch (i & 3) {
          case 0: a0 = MFMA(t[i >> 2][0], pA, a0); break;
          case 1: a1 = MFMA(t[i >> 2][1], pA, a1); break;
          case 2: a2 = MFMA(t[i >> 2][2], pA, a2); break;
          default: a3 = MFMA(t[i >> 2][3], pA, a3); break;
        }
        FENCE();
        eB[2 * i] = __builtin_amdgcn_exp2f(fmaf(sB[2 * i], c, -mcB));
        eB[2 * i + 1] = __builtin_amdgcn_exp2f(fmaf(sB[2 * i + 1], c, -mcB));
      }
      FENCE();
      if (n_valid < 32) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (8 * (v >> 2) + 4 * g + (v & 3) >= n_valid) eB[v] = 0.f;
      }
      {
        float ps = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) ps += eB[v];
        lB += ps;
      }
      const bf16x8 pb0 = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(eB[0], eB[1]), pack_bf16(eB[2], eB[3]),
                                                                pack_bf16(eB[4], eB[5]), pack_bf16(eB[6], eB[7])));
      const bf16x8 pb1 = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(eB[8], eB[9]), pack_bf16(eB[10], eB[11]),
                                                                pack_bf16(eB[12], eB[13]), pack_bf16(eB[14], eB[15])));
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 pB = kk ? pb1 : pb0;
        b0 = MFMA(t[kk][0], pB, b0);
        b1 = MFMA(t[kk][1], pB, b1);
        b2 = MFMA(t[kk][2], pB, b2);
        b3 = MFMA(t[kk][3], pB, b3);
      }
      if (h == 1) {
        if (it + 1 < n_blocks) { STAGE((it + 1) & 1) }
        __syncthreads();
        r = nr; pos = npos; start = nstart; len = nlen;
        fetched = false;
      }
    }
    if (!raise) break;
    // ---------------- cold path: raise the references to the running maxima ----------------
    {
      const float newA = fmaxf(mrunA, __shfl_xor(mrunA, 32, 64));
      const float newB = fmaxf(mrunB, __shfl_xor(mrunB, 32, 64));
      const float alA = __builtin_amdgcn_exp2f((mrefA - newA) * c);   // 0 on the first pass (m_ref = -inf)
      const float alB = __builtin_amdgcn_exp2f((mrefB - newB) * c);
      lA *= alA;
      lB *= alB;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        a0[v] *= alA; a1[v] *= alA; a2[v] *= alA; a3[v] *= alA;
        b0[v] *= alB; b1[v] *= alB; b2[v] *= alB; b3[v] *= alB;
      }
      mrefA = newA;
      mrefB = newB;
    }
  }
#undef FENCE
#undef PIN

  // ---- epilogue: two passes (block A, block B) through a per-wave LDS staging area
  uint16_t* st = smem + wave * 32 * LSTR;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const float l_run = half ? lB : lA;
    const float inv = 1.f / (l_run + __shfl_xor(l_run, 32, 64));
    if (half == 0) { STORE_TILE(0, a0) STORE_TILE(1, a1) STORE_TILE(2, a2) STORE_TILE(3, a3) }
    else { STORE_TILE(0, b0) STORE_TILE(1, b1) STORE_TILE(2, b2) STORE_TILE(3, b3) }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = (lane >> 4) + 4 * i;
      const int qrow = 64 * wave + 32 * half + row;
      if (qrow < w.n_rows)
        *(uint4*)(O + (unsigned)(w.row0 + qrow) * row_stride + (lane & 15) * 8) =
            *(const uint4*)(st + row * LSTR + (lane & 15) * 8);
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// Ping-pong variant for the dense and core-set segments.  Eight wavefronts of 32 query rows;
// the SIMD that hosts wavefronts w and w+4 sees them in opposite phases:
//     M phase   O^T += V^T P^T of the previous key block, then S^T = K Q^T of the current one
//               (32 matrix instructions, all LDS fragment reads)
//     V phase   softmax arithmetic of the current block (exp, sums, bf16 packing), plus the
//               global -> LDS staging two blocks ahead
// with a workgroup barrier at every phase change and the upper four wavefronts started half an
// iteration late, so the matrix pipe of a SIMD is fed by one wavefront while the vector pipe
// works for the other.  Softmax uses the lazy per-query reference (see REF_SLACK above); the
// O rescale runs only when a reference has to be raised.  Four LDS stages keep the block being
// written apart from the two being read by either group.
// ------------------------------------------------------------------------------------------
namespace {
constexpr int PP_BUFS = 4;
constexpr int PP_LDS_BYTES = PP_BUFS * STAGE_ELEMS * 2;
}  // namespace

#ifdef VORTA_PP_TIMING   // debug build: per-phase wall-clock (100 MHz ticks) of wavefronts 0 and 4 of block 0
__device__ long long g_pp_timing[2][16];
#define PP_T_DECL long long tacc_[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; long long tprev_ = __builtin_amdgcn_s_memrealtime();
#define PP_T_MARK(i_) { const long long now_ = __builtin_amdgcn_s_memrealtime(); tacc_[i_] += now_ - tprev_; tprev_ = now_; }
#define PP_T_DUMP if (blockIdx.x == 0 && lane == 0 && (wave == 0 || wave == 4)) { for (int i = 0; i < 12; ++i) g_pp_timing[wave >> 2][i] = tacc_[i]; g_pp_timing[wave >> 2][15] = n_blocks; }
#else
#define PP_T_DECL
#define PP_T_MARK(i_)
#define PP_T_DUMP
#endif

__global__ __launch_bounds__(512, 1) void attn_bf16_pp_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int STG_ROWS = 32, STG_PASSES = 2;
  const WorkItem w = decode_item<BM2, D>(a, blockIdx.x);
  const uint16_t* Q = (const uint16_t*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const uint16_t* K = (const uint16_t*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const uint16_t* V = (const uint16_t*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  uint16_t* O = (uint16_t*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  const unsigned row_stride = (unsigned)w.row_stride;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int grp = wave >> 2;

  bf16x8 qf[8];
  {
    const unsigned qrow = w.row0 + min(32 * wave + l32, w.n_rows - 1);
    const uint16_t* qp = Q + qrow * row_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * ks));
  }

  const int ld_row = tid >> 4, ld_col = (tid & 15) * 8;
  uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
  auto run_start = [&](int r) { return w.runs ? w.runs[2 * r] : 0; };
  auto run_len = [&](int r) { return w.runs ? w.runs[2 * r + 1] : w.single_len; };
  int n_blocks = 0;
  for (int r = 0; r < w.n_runs; ++r) n_blocks += (run_len(r) + BN - 1) / BN;

  // fetch cursor (block being requested) and compute cursor (block being used)
  int fr = 0, fpos = 0, fstart = run_start(0), flen = run_len(0);
  int cr = 0, cpos = 0, clen = flen;
#define FETCH_NEXT()                                                     \
  {                                                                      \
    FETCH(fstart, flen, fpos)                                            \
    fpos += BN;                                                          \
    if (fpos >= flen) {                                                  \
      ++fr;                                                              \
      fpos = 0;                                                          \
      if (fr < w.n_runs) { fstart = run_start(fr); flen = run_len(fr); } \
    }                                                                    \
  }
  FETCH_NEXT()
  STAGE(0)
  if (n_blocks > 1) {
    FETCH_NEXT()
    STAGE(1)
  }
  if (n_blocks > 2) { FETCH_NEXT() }          // block 2 waits in registers
  __syncthreads();
  if (grp == 1) __syncthreads();              // upper group runs half an iteration behind

  f32x16 o0, o1, o2, o3;
#pragma unroll
  for (int v = 0; v < 16; ++v) { o0[v] = 0.f; o1[v] = 0.f; o2[v] = 0.f; o3[v] = 0.f; }
  const float c = a.scale * 1.4426950408889634f;
  const float slack = REF_SLACK / c;
  float m_ref = -INFINITY, m_run = -INFINITY, l_run = 0.f;
  bf16x8 pf[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) pf[i] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));

  const uint16_t* k_rd = smem + l32 * LSTR + 8 * g;
  const int t16 = lane & 15, blk = lane >> 4;
  const uint16_t* v_rd = smem + KTILE + (4 * g + (t16 >> 2)) * VSTR + 16 * (blk & 1) + 4 * (t16 & 3);

  f32x16 oacc[4] = {o0, o1, o2, o3};
  f32x16 sacc[2];
  bf16x8 frag[32];            // fragment of matrix-instruction slot i: slots 0..15 = V^T for PV, 16..31 = K for QK
  // LDS fragment of slot i.  PV slot (kk, dt) = (i / 4, i % 4) of stage `sv`; QK slot (ks, sb) = ((i - 16) / 2, i % 2)
  // of stage `sk`.
#define LOAD_SLOT(i_, vp_, kp_)                                                                   \
  {                                                                                               \
    if ((i_) < 16) {                                                                              \
      const uint16_t* a_ = (vp_) + 16 * ((i_) >> 2) * VSTR + 32 * ((i_)&3);                       \
      frag[i_] = read_vt(a_, a_ + 8 * VSTR);                                                        \
    } else {                                                                                      \
      frag[i_] = lds_frag((kp_) + 32 * ((i_)&1) * LSTR + 16 * (((i_)-16) >> 1));                    \
    }                                                                                             \
  }
#define MFMA_SLOT(i_)                                                                             \
  {                                                                                               \
    if ((i_) < 16) oacc[(i_)&3] = MFMA(frag[i_], pf[(i_) >> 2], oacc[(i_)&3]);                      \
    else sacc[(i_)&1] = MFMA(frag[i_], qf[((i_)-16) >> 1], sacc[(i_)&1]);                           \
  }
  PP_T_DECL
  constexpr int LEAD = 8;   // fragments requested this many matrix instructions ahead of their use

  // V phase of block j: softmax arithmetic on sacc -> pf, staging two blocks ahead, and the
  // first LEAD fragment requests of the next M phase (PV of this block) so they are in flight
  // across the barrier.
  auto v_phase = [&](int j) {
    f32x16& s0 = sacc[0];
    f32x16& s1 = sacc[1];
    const int n_valid = min(BN, clen - cpos);
    cpos += BN;
    if (cpos >= clen) {
      ++cr;
      cpos = 0;
      if (cr < w.n_runs) clen = run_len(cr);
    }
    // rows past the end of a run repeat its last row: they cannot raise a maximum, only
    // their probabilities are zeroed below
    float mx = max3(s0[0], s1[0], s0[1]);
    mx = max3(mx, s1[1], s0[2]);
#pragma unroll
    for (int v = 2; v < 15; ++v) mx = max3(mx, s1[v], s0[v + 1]);
    mx = fmaxf(mx, s1[15]);
    m_run = fmaxf(m_run, mx);
    PP_T_MARK(5)
    if (__any(mx > m_ref + slack)) {
      const float m_new = fmaxf(m_run, __shfl_xor(m_run, 32, 64));
      const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c);   // 0 the first time
      l_run *= alpha;
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[d][v] *= alpha;
      m_ref = m_new;
    }
    PP_T_MARK(6)
    const float mc = m_ref * c;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s0[v] = __builtin_amdgcn_exp2f(fmaf(s0[v], c, -mc));
      s1[v] = __builtin_amdgcn_exp2f(fmaf(s1[v], c, -mc));
    }
    if (n_valid < BN) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 8 * (v >> 2) + 4 * g + (v & 3);
        if (key >= n_valid) s0[v] = 0.f;
        if (key + 32 >= n_valid) s1[v] = 0.f;
      }
    }
    float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) { ps0 += s0[v]; ps1 += s1[v]; }
    l_run += ps0 + ps1;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint4 u0, u1;
      u0.x = pack_bf16(s0[8 * h + 0], s0[8 * h + 1]); u0.y = pack_bf16(s0[8 * h + 2], s0[8 * h + 3]);
      u0.z = pack_bf16(s0[8 * h + 4], s0[8 * h + 5]); u0.w = pack_bf16(s0[8 * h + 6], s0[8 * h + 7]);
      u1.x = pack_bf16(s1[8 * h + 0], s1[8 * h + 1]); u1.y = pack_bf16(s1[8 * h + 2], s1[8 * h + 3]);
      u1.z = pack_bf16(s1[8 * h + 4], s1[8 * h + 5]); u1.w = pack_bf16(s1[8 * h + 6], s1[8 * h + 7]);
      pf[h] = __builtin_bit_cast(bf16x8, u0);
      pf[2 + h] = __builtin_bit_cast(bf16x8, u1);
    }
    PP_T_MARK(7)
    if (j + 2 < n_blocks) { STAGE((j + 2) & 3) }
    PP_T_MARK(8)
    if (j + 3 < n_blocks) { FETCH_NEXT() }
    PP_T_MARK(9)
    const uint16_t* vp = v_rd + (j & 3) * STAGE_ELEMS;
#pragma unroll
    for (int i = 0; i < LEAD; ++i) LOAD_SLOT(i, vp, vp)
  };

  // ---- block 0: QK only
  {
    const uint16_t* kp = k_rd;
#pragma unroll
    for (int v = 0; v < 16; ++v) { sacc[0][v] = 0.f; sacc[1][v] = 0.f; }
#pragma unroll
    for (int i = 16; i < 32; ++i) LOAD_SLOT(i, kp, kp)
#pragma unroll
    for (int i = 16; i < 32; ++i) MFMA_SLOT(i)
  }
  __syncthreads();
  v_phase(0);
  __syncthreads();
  // ---- blocks 1 .. n-1: PV of the previous block, then QK of this one, one fragment stream
  for (int j = 1; j < n_blocks; ++j) {
    PP_T_MARK(0)
    const uint16_t* vp = v_rd + ((j - 1) & 3) * STAGE_ELEMS;
    const uint16_t* kp = k_rd + (j & 3) * STAGE_ELEMS;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if (i == 16) {
#pragma unroll
        for (int v = 0; v < 16; ++v) { sacc[0][v] = 0.f; sacc[1][v] = 0.f; }
      }
      MFMA_SLOT(i)
      if (i + LEAD < 32) LOAD_SLOT(i + LEAD, vp, kp)
      __builtin_amdgcn_sched_barrier(0);
    }
    PP_T_MARK(1)
    __syncthreads();
    PP_T_MARK(2)
    v_phase(j);
    PP_T_MARK(3)
    __syncthreads();
    PP_T_MARK(4)
  }
  // ---- PV of the last block
  {
    const uint16_t* vp = v_rd + ((n_blocks - 1) & 3) * STAGE_ELEMS;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      MFMA_SLOT(i)
      if (i + LEAD < 16) LOAD_SLOT(i + LEAD, vp, vp)
    }
  }
  __syncthreads();
  __syncthreads();
  if (grp == 0) __syncthreads();
  PP_T_DUMP
  o0 = oacc[0]; o1 = oacc[1]; o2 = oacc[2]; o3 = oacc[3];
#undef LOAD_SLOT
#undef MFMA_SLOT
#undef FETCH_NEXT

  // ---- epilogue: normalise, transpose through LDS, store whole rows
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  uint16_t* st = smem + wave * 32 * LSTR;
  STORE_TILE(0, o0) STORE_TILE(1, o1) STORE_TILE(2, o2) STORE_TILE(3, o3)
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (lane >> 4) + 4 * i;
    if (32 * wave + row < w.n_rows)
      *(uint4*)(O + (unsigned)(w.row0 + 32 * wave + row) * row_stride + (lane & 15) * 8) =
          *(const uint4*)(st + row * LSTR + (lane & 15) * 8);
  }
}

// ------------------------------------------------------------------------------------------
// Interleaved variant for the dense and core-set segments.  Measurements on gfx950: vector
// instructions issued by the SAME wavefront right behind a matrix instruction run in its shadow
// (about six per v_mfma_f32_32x32x16_bf16, an exp counting double), while vector work of
// another wavefront on the SIMD mostly serialises with it.  So every wavefront software-
// pipelines its own loop over 32-key sub-steps t:
//     matrix pipe   QK of sub-step t+1 (8 instr.)  then  PV of sub-step t-1 (8 instr.)
//     vector pipe   exp / sum / bf16 packing of sub-step t, then the row maximum of t+1,
//                   a few instructions behind each matrix instruction
// with LDS fragments requested IL_LEAD matrix instructions ahead (the first ones of a sub-step
// at the end of the previous one).  Eight wavefronts of 32 query rows share 64-key LDS stages,
// three buffers, one barrier per stage.  Softmax uses the lazy per-query reference (REF_SLACK).
// ------------------------------------------------------------------------------------------
namespace {
constexpr int IL_BUFS = 3;
constexpr int IL_LDS_BYTES = IL_BUFS * STAGE_ELEMS * 2;
constexpr int IL_LEAD = 4;
}  // namespace

__global__ __launch_bounds__(512, 1) void attn_bf16_il_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int STG_ROWS = 32, STG_PASSES = 2;
  const WorkItem w = decode_item<BM2, D>(a, blockIdx.x);
  const uint16_t* Q = (const uint16_t*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const uint16_t* K = (const uint16_t*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const uint16_t* V = (const uint16_t*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  uint16_t* O = (uint16_t*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  const unsigned row_stride = (unsigned)w.row_stride;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;

  bf16x8 qf[8];
  {
    const unsigned qrow = w.row0 + min(32 * wave + l32, w.n_rows - 1);
    const uint16_t* qp = Q + qrow * row_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * ks));
  }

  const int ld_row = tid >> 4, ld_col = (tid & 15) * 8;
  uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
  auto run_start = [&](int r) { return w.runs ? w.runs[2 * r] : 0; };
  auto run_len = [&](int r) { return w.runs ? w.runs[2 * r + 1] : w.single_len; };
  int n_blocks = 0;
  for (int r = 0; r < w.n_runs; ++r) n_blocks += (run_len(r) + BN - 1) / BN;

  int fr = 0, fpos = 0, fstart = run_start(0), flen = run_len(0);   // fetch cursor
  int cr = 0, cpos = 0, clen = flen;                                 // compute cursor
#define FETCH_NEXT()                                                     \
  {                                                                      \
    FETCH(fstart, flen, fpos)                                            \
    fpos += BN;                                                          \
    if (fpos >= flen) {                                                  \
      ++fr;                                                              \
      fpos = 0;                                                          \
      if (fr < w.n_runs) { fstart = run_start(fr); flen = run_len(fr); } \
    }                                                                    \
  }
  FETCH_NEXT()
  STAGE(0)
  if (n_blocks > 1) { FETCH_NEXT() }          // stage 1 waits in registers
  __syncthreads();

  f32x16 oacc[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[d][v] = 0.f;
  const float c = a.scale * 1.4426950408889634f;
  const float slack = REF_SLACK / c;
  float m_ref = -INFINITY, m_run = -INFINITY, l_run = 0.f;

  const lds_ptr k_rd = (lds_ptr)(smem + l32 * LSTR + 8 * g);
  const int t16 = lane & 15, blk = lane >> 4;
  const lds_ptr v_rd = (lds_ptr)(smem + KTILE + (4 * g + (t16 >> 2)) * VSTR + 16 * (blk & 1) + 4 * (t16 & 3));

  // scores of sub-step 0 and the first fragments of sub-step 0's matrix work (QK of sub-step 1)
  f32x16 s_even, s_odd;     // scores of even / odd sub-steps
#pragma unroll
  for (int v = 0; v < 16; ++v) s_even[v] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) s_even = MFMA(lds_frag3(k_rd + 16 * ks), qf[ks], s_even);
  float mx_cur = max16(s_even);
  bf16x8 pre[IL_LEAD];
#pragma unroll
  for (int i = 0; i < IL_LEAD; ++i) pre[i] = lds_frag3(k_rd + 32 * LSTR + 16 * i);
  bf16x8 p_prev[2];
  p_prev[0] = p_prev[1] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));

  // One 32-key sub-step.  kq: K fragments of sub-step t+1; vq: V fragments of sub-step t-1;
  // kn: K fragments of sub-step t+2 (first IL_LEAD requested at the end); n_valid: valid keys of
  // sub-step t.  FAST pins the instruction order; the other copy handles run tails.
  auto substep = [&](auto fast_tag, f32x16& s_cur, f32x16& s_next, lds_ptr kq, lds_ptr vq, int n_valid) {
    constexpr bool FAST = decltype(fast_tag)::value;
#define IL_FENCE() do { if (FAST) __builtin_amdgcn_sched_barrier(0); } while (0)
    m_run = fmaxf(m_run, mx_cur);
    // Raising the reference: this sub-step's exponentials use the new one at once; the
    // accumulators are rescaled only after PV of the previous sub-step (old reference) is in.
    const bool raised = __any(mx_cur > m_ref + slack);
    float alpha = 1.f;
    if (raised) {
      const float m_new = fmaxf(m_run, __shfl_xor(m_run, 32, 64));
      alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c);   // 0 the first time
      l_run *= alpha;
      m_ref = m_new;
    }
    const float mc = m_ref * c;
    bf16x8 f[16];
#pragma unroll
    for (int i = 0; i < IL_LEAD; ++i) f[i] = pre[i];
#pragma unroll
    for (int v = 0; v < 16; ++v) s_next[v] = 0.f;
    unsigned u[8];
    float ps = 0.f, mxn = 0.f;
    IL_FENCE();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      // ---- matrix instruction of slot i
      if (i < 8) s_next = MFMA(f[i], qf[i], s_next);
      else oacc[(i - 8) & 3] = MFMA(f[i], p_prev[(i - 8) >> 2], oacc[(i - 8) & 3]);
      // ---- fragment request IL_LEAD slots ahead
      if (i + IL_LEAD < 8) {
        f[i + IL_LEAD] = lds_frag3(kq + 16 * (i + IL_LEAD));
      } else if (i + IL_LEAD < 16) {
        const int sl = i + IL_LEAD - 8;
        const lds_ptr ap = vq + 16 * (sl >> 2) * VSTR + 32 * (sl & 3);
        f[i + IL_LEAD] = read_vt3(ap, ap + 8 * VSTR);
      }
      // ---- vector work in the shadow
      if (i < 8) {
        s_cur[2 * i] = __builtin_amdgcn_exp2f(fmaf(s_cur[2 * i], c, -mc));
        s_cur[2 * i + 1] = __builtin_amdgcn_exp2f(fmaf(s_cur[2 * i + 1], c, -mc));
        if (!FAST) {
          if (8 * ((2 * i) >> 2) + 4 * g + ((2 * i) & 3) >= n_valid) s_cur[2 * i] = 0.f;
          if (8 * ((2 * i + 1) >> 2) + 4 * g + ((2 * i + 1) & 3) >= n_valid) s_cur[2 * i + 1] = 0.f;
        }
      } else if (i < 12) {
        const int b4 = 4 * (i - 8);
        ps += (s_cur[b4] + s_cur[b4 + 1]) + (s_cur[b4 + 2] + s_cur[b4 + 3]);
        u[2 * (i - 8)] = pack_bf16(s_cur[b4], s_cur[b4 + 1]);
        u[2 * (i - 8) + 1] = pack_bf16(s_cur[b4 + 2], s_cur[b4 + 3]);
      } else {
        const int b4 = 4 * (i - 12);
        const float m4 = max3(s_next[b4], s_next[b4 + 1], fmaxf(s_next[b4 + 2], s_next[b4 + 3]));
        mxn = (i == 12) ? m4 : fmaxf(mxn, m4);
      }
      IL_FENCE();
    }
    if (raised) {
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[d][v] *= alpha;
    }
    l_run += ps;
    p_prev[0] = __builtin_bit_cast(bf16x8, make_uint4(u[0], u[1], u[2], u[3]));
    p_prev[1] = __builtin_bit_cast(bf16x8, make_uint4(u[4], u[5], u[6], u[7]));
    mx_cur = mxn;
#undef IL_FENCE
  };
  auto request_pre = [&](lds_ptr kn) {
#pragma unroll
    for (int i = 0; i < IL_LEAD; ++i) pre[i] = lds_frag3(kn + 16 * i);
  };

  for (int it = 0; it < n_blocks; ++it) {
    const int n_valid = min(BN, clen - cpos);
    cpos += BN;
    if (cpos >= clen) {
      ++cr;
      cpos = 0;
      if (cr < w.n_runs) clen = run_len(cr);
    }
    const int b_prev = (it + IL_BUFS - 1) % IL_BUFS, b_cur = it % IL_BUFS, b_next = (it + 1) % IL_BUFS;
    // ---- sub-step 2 it: QK of keys [32, 64) of this stage, PV of the previous stage's keys [32, 64)
    {
      const lds_ptr kq = opaque(k_rd + b_cur * STAGE_ELEMS + 32 * LSTR);
      const lds_ptr vq = opaque(it ? v_rd + b_prev * STAGE_ELEMS + 32 * VSTR : v_rd);   // it = 0: P is zero, any finite V
      if (n_valid >= 32) substep(std::true_type{}, s_even, s_odd, kq, vq, 32);
      else substep(std::false_type{}, s_even, s_odd, kq, vq, n_valid);
    }
    // publish the next stage, request the one after
    if (it + 1 < n_blocks) { STAGE(b_next) }
    __syncthreads();
    if (it + 2 < n_blocks) { FETCH_NEXT() }
    const lds_ptr k_next = opaque(k_rd + b_next * STAGE_ELEMS);
    request_pre(k_next);
    // ---- sub-step 2 it + 1: QK of keys [0, 32) of the next stage, PV of this stage's keys [0, 32)
    {
      const lds_ptr kq = k_next;
      const lds_ptr vq = opaque(v_rd + b_cur * STAGE_ELEMS);
      if (n_valid >= 64) substep(std::true_type{}, s_odd, s_even, kq, vq, 32);
      else substep(std::false_type{}, s_odd, s_even, kq, vq, n_valid - 32);
    }
    request_pre(k_next + 32 * LSTR);
  }
#undef FETCH_NEXT
  // ---- PV of the last sub-step: keys [32, 64) of the last stage
  {
    const lds_ptr vq = opaque(v_rd + ((n_blocks - 1) % IL_BUFS) * STAGE_ELEMS + 32 * VSTR);
#pragma unroll
    for (int sl = 0; sl < 8; ++sl) {
      const lds_ptr ap = vq + 16 * (sl >> 2) * VSTR + 32 * (sl & 3);
      oacc[sl & 3] = MFMA(read_vt3(ap, ap + 8 * VSTR), p_prev[sl >> 2], oacc[sl & 3]);
    }
  }
  __syncthreads();

  // ---- epilogue: normalise, transpose through LDS, store whole rows
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  uint16_t* st = smem + wave * 32 * LSTR;
  STORE_TILE(0, oacc[0]) STORE_TILE(1, oacc[1]) STORE_TILE(2, oacc[2]) STORE_TILE(3, oacc[3])
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (lane >> 4) + 4 * i;
    if (32 * wave + row < w.n_rows)
      *(uint4*)(O + (unsigned)(w.row0 + 32 * wave + row) * row_stride + (lane & 15) * 8) =
          *(const uint4*)(st + row * LSTR + (lane & 15) * 8);
  }
}

static int g_long_variant = getenv("VORTA_LONG_VARIANT") ? atoi(getenv("VORTA_LONG_VARIANT")) : 0;   // experiment switch

static int set_lds_limit(const void* kernel, const char* name) {
  hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e != hipSuccess) return fail(VORTA_EHIP, "hipFuncSetAttribute(%s, %d B LDS): %s", name, LDS_BYTES, hipGetErrorString(e));
  return VORTA_OK;
}

int launch_attention_bf16(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream) {
  static std::once_flag once;
  static int attr_rc = VORTA_OK;
  std::call_once(once, [] {
    attr_rc = set_lds_limit((const void*)attn_bf16_kernel<4>, "attn_bf16_kernel<4>");
    if (!attr_rc) attr_rc = set_lds_limit((const void*)attn_bf16_kernel<8>, "attn_bf16_kernel<8>");
    if (!attr_rc) attr_rc = set_lds_limit((const void*)attn_bf16_m64_kernel, "attn_bf16_m64_kernel");
    if (!attr_rc) {
      hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_pp_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, PP_LDS_BYTES);
      if (e != hipSuccess) attr_rc = fail(VORTA_EHIP, "hipFuncSetAttribute(attn_bf16_pp_kernel): %s", hipGetErrorString(e));
    }
    if (!attr_rc) {
      hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_il_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, IL_LDS_BYTES);
      if (e != hipSuccess) attr_rc = fail(VORTA_EHIP, "hipFuncSetAttribute(attn_bf16_il_kernel): %s", hipGetErrorString(e));
    }
  });
  if (attr_rc) return attr_rc;
  // dense + core-set heads: 256-row workgroups; window heads: 128-row workgroups (one tile each)
  RouteLists long_rl = rl, win_rl = rl;
  long_rl.count[1] = 0;
  win_rl.count[0] = win_rl.count[2] = 0;
  AttnArgs a;
  if (int rc = fill_attn_args(p, long_rl, io, BM2, &a)) return rc;
  if (a.end_text > 0) {
    if (g_long_variant == 1)
      hipLaunchKernelGGL(attn_bf16_m64_kernel, dim3(a.end_text), dim3(256), LDS_BYTES, (hipStream_t)stream, a);
    else if (g_long_variant == 2)
      hipLaunchKernelGGL(attn_bf16_pp_kernel, dim3(a.end_text), dim3(512), PP_LDS_BYTES, (hipStream_t)stream, a);
    else if (g_long_variant == 3)
      hipLaunchKernelGGL(attn_bf16_il_kernel, dim3(a.end_text), dim3(512), IL_LDS_BYTES, (hipStream_t)stream, a);
    else
      hipLaunchKernelGGL(attn_bf16_kernel<8>, dim3(a.end_text), dim3(512), LDS_BYTES, (hipStream_t)stream, a);
  }
  if (int rc = fill_attn_args(p, win_rl, io, BM, &a)) return rc;
  if (a.end_text > 0) hipLaunchKernelGGL(attn_bf16_kernel<4>, dim3(a.end_text), dim3(256), LDS_BYTES, (hipStream_t)stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(VORTA_EHIP, "launch of attn_bf16 kernels: %s", hipGetErrorString(e));
  return VORTA_OK;
}

}  // namespace vorta

#ifdef VORTA_PP_TIMING
extern "C" int vorta_debug_pp_timing(long long* out16) {
  return hipMemcpyFromSymbol(out16, HIP_SYMBOL(vorta::g_pp_timing), sizeof(long long) * 32) == hipSuccess ? 0 : -6;
}
#endif
