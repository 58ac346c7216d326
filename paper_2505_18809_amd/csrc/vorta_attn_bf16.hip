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
constexpr int LSTR = 136;       // LDS row stride in elements: 256 B of data + 16 B pad
constexpr int TILE = BN * LSTR; // elements of one K (or V) block in LDS
constexpr int LDS_BYTES = 2 * 2 * TILE * 2;
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

__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const WorkItem w = decode_item<BM, D>(a, blockIdx.x);
  const uint16_t* Q = (const uint16_t*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const uint16_t* K = (const uint16_t*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const uint16_t* V = (const uint16_t*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  uint16_t* O = (uint16_t*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;

  // Q^T fragments: lane = query (l32), 8 consecutive dims per 16-wide k slice
  bf16x8 qf[8];
  {
    const int qrow = w.row0 + min(32 * wave + l32, w.n_rows - 1);
    const uint16_t* qp = Q + (long)qrow * w.row_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * ks));
  }

  // global -> LDS staging: thread moves the 16-byte chunk (tid & 15) of rows (tid >> 4) + 16 i
  const int ld_row = tid >> 4, ld_col = (tid & 15) * 8;
  uint4 kreg[4], vreg[4];
  auto fetch = [&](int start, int len, int pos) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = min(pos + ld_row + 16 * i, len - 1);   // rows past the run repeat its last row
      const long off = (long)(start + r) * w.row_stride + ld_col;
      kreg[i] = *(const uint4*)(K + off);
      vreg[i] = *(const uint4*)(V + off);
    }
  };
  auto stage = [&](int buf) {
    uint16_t* kb = smem + buf * 2 * TILE + ld_row * LSTR + ld_col;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(uint4*)(kb + 16 * i * LSTR) = kreg[i];
      *(uint4*)(kb + TILE + 16 * i * LSTR) = vreg[i];
    }
  };
  auto run_start = [&](int r) { return w.runs ? w.runs[2 * r] : 0; };
  auto run_len = [&](int r) { return w.runs ? w.runs[2 * r + 1] : w.single_len; };

  int n_blocks = 0;
  for (int r = 0; r < w.n_runs; ++r) n_blocks += (run_len(r) + BN - 1) / BN;

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = a.scale * 1.4426950408889634f;

  int r = 0, pos = 0, start = run_start(0), len = run_len(0);
  fetch(start, len, 0);
  stage(0);
  __syncthreads();

  // per-lane LDS read offsets
  const uint16_t* k_rd = smem + l32 * LSTR + 8 * g;
  const int t16 = lane & 15, blk = lane >> 4;
  const uint16_t* v_rd = smem + TILE + (4 * g + (t16 >> 2)) * LSTR + 16 * (blk & 1) + 4 * (t16 & 3);

  for (int it = 0; it < n_blocks; ++it) {
    // cursor of the next block
    int nr = r, npos = pos + BN, nstart = start, nlen = len;
    if (npos >= len) {
      nr = r + 1;
      npos = 0;
      if (nr < w.n_runs) { nstart = run_start(nr); nlen = run_len(nr); }
    }
    const bool has_next = it + 1 < n_blocks;
    if (has_next) fetch(nstart, nlen, npos);

    const int n_valid = min(BN, len - pos);
    const int buf_off = (it & 1) * 2 * TILE;

    // ---- S^T = K Q^T for keys [0,32) and [32,64) of the block
    f32x16 s0, s1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { s0[v] = 0.f; s1[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a0 = __builtin_bit_cast(bf16x8, *(const uint4*)(k_rd + buf_off + 16 * ks));
      const bf16x8 a1 = __builtin_bit_cast(bf16x8, *(const uint4*)(k_rd + buf_off + 32 * LSTR + 16 * ks));
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[ks], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[ks], s1, 0, 0, 0);
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
    float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, fmaxf(s0[v], s1[v]));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    if (__any(m_new > m_run)) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
      m_run = m_new;
    }
    const float mc = m_run * c;
    float psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s0[v] = __builtin_amdgcn_exp2f(fmaf(s0[v], c, -mc));
      s1[v] = __builtin_amdgcn_exp2f(fmaf(s1[v], c, -mc));
      psum += s0[v] + s1[v];
    }
    l_run += psum;

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
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const uint16_t* vp = v_rd + buf_off + 16 * kk * LSTR + 32 * dt;
        const bf16x8 vt = read_vt(vp, vp + 8 * LSTR);
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt, pf[kk], o[dt], 0, 0, 0);
      }
    }

    if (has_next) stage((it + 1) & 1);
    __syncthreads();
    r = nr; pos = npos; start = nstart; len = nlen;
  }

  // ---- epilogue: normalise, transpose through LDS, store whole rows
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  uint16_t* st = smem + wave * 32 * LSTR;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      uint2 u;
      u.x = pack_bf16(o[dt][4 * q4] * inv, o[dt][4 * q4 + 1] * inv);
      u.y = pack_bf16(o[dt][4 * q4 + 2] * inv, o[dt][4 * q4 + 3] * inv);
      *(uint2*)(st + l32 * LSTR + 32 * dt + 8 * q4 + 4 * g) = u;
    }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (lane >> 4) + 4 * i;
    if (32 * wave + row < w.n_rows)
      *(uint4*)(O + (long)(w.row0 + 32 * wave + row) * w.row_stride + (lane & 15) * 8) =
          *(const uint4*)(st + row * LSTR + (lane & 15) * 8);
  }
}

int launch_attention_bf16(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream) {
  AttnArgs a;
  if (int rc = fill_attn_args(p, rl, io, BM, &a)) return rc;
  if (a.end_text == 0) return VORTA_OK;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute((const void*)attn_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   LDS_BYTES);
  });
  if (attr_err != hipSuccess)
    return fail(VORTA_EHIP, "hipFuncSetAttribute(dynamic LDS %d): %s", LDS_BYTES, hipGetErrorString(attr_err));
  hipLaunchKernelGGL(attn_bf16_kernel, dim3(a.end_text), dim3(256), LDS_BYTES, (hipStream_t)stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(VORTA_EHIP, "launch of attn_bf16_kernel: %s", hipGetErrorString(e));
  return VORTA_OK;
}

}  // namespace vorta
