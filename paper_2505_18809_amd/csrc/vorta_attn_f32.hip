// fp32 routed attention for gfx950: the exact-precision path (small layers, 1e-5 parity).
// One thread owns one query row (q and the output accumulator live in registers); a
// workgroup of one wavefront streams the item's key runs through LDS 32 keys at a time and
// every lane reads the same K / V element at once (an LDS broadcast).  Online softmax in
// fp32 with precise expf.  Throughput is not a goal of this kernel; the bf16 MFMA kernel is
// the fast path.
#include <hip/hip_runtime.h>

#include "vorta_attn_common.h"

namespace vorta {

template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(const AttnArgs a) {
  constexpr int BM = 64, BN = 32;
  __shared__ float sK[BN][D];
  __shared__ float sV[BN][D];
  const WorkItem w = decode_item<BM, D>(a, blockIdx.x);
  const float* Q = (const float*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const float* K = (const float*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const float* V = (const float*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  float* O = (float*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  if (w.n_rows <= 0) return;       // q-block past the end of a clipped tile
  const int t = threadIdx.x;
  const long my_row = w.row0 + min(t, w.n_rows - 1);

  float q[D], o[D];
  {
    const float4* src = (const float4*)(Q + my_row * w.row_stride);
#pragma unroll
    for (int c = 0; c < D / 4; ++c) {
      const float4 x = src[c];
      q[4 * c] = x.x; q[4 * c + 1] = x.y; q[4 * c + 2] = x.z; q[4 * c + 3] = x.w;
    }
  }
#pragma unroll
  for (int c = 0; c < D; ++c) o[c] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int r = 0; r < w.n_runs; ++r) {
    const int start = w.runs ? w.runs[2 * r] : 0;
    const int len = w.runs ? w.runs[2 * r + 1] : w.single_len;
    for (int pos = 0; pos < len; pos += BN) {
      const int n_valid = min(BN, len - pos);
      __syncthreads();
      for (int c = t; c < BN * D / 4; c += 64) {
        const int j = c / (D / 4), e = c - j * (D / 4);
        const long row = start + pos + min(j, n_valid - 1);   // rows past the run repeat its last row
        ((float4*)&sK[j][0])[e] = ((const float4*)(K + row * w.row_stride))[e];
        ((float4*)&sV[j][0])[e] = ((const float4*)(V + row * w.row_stride))[e];
      }
      __syncthreads();
      float s[BN];
      float mt = -INFINITY;
#pragma unroll
      for (int j = 0; j < BN; ++j) {
        float dot = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) dot = fmaf(q[c], sK[j][c], dot);
        s[j] = j < n_valid ? dot * a.scale : -INFINITY;
        mt = fmaxf(mt, s[j]);
      }
      const float m_new = fmaxf(m, mt);
      const float alpha = expf(m - m_new);
      l *= alpha;
#pragma unroll
      for (int c = 0; c < D; ++c) o[c] *= alpha;
#pragma unroll
      for (int j = 0; j < BN; ++j) {
        const float pj = expf(s[j] - m_new);
        l += pj;
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = fmaf(pj, sV[j][c], o[c]);
      }
      m = m_new;
    }
  }
  if (t < w.n_rows) {
    const float inv = 1.f / l;
    float4* dst = (float4*)(O + my_row * w.row_stride);
#pragma unroll
    for (int c = 0; c < D / 4; ++c)
      dst[c] = make_float4(o[4 * c] * inv, o[4 * c + 1] * inv, o[4 * c + 2] * inv, o[4 * c + 3] * inv);
  }
}

int launch_attention_f32(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream) {
  AttnArgs a;
  if (int rc = fill_attn_args(p, rl, io, 64, WIN_ALL, &a)) return rc;
  if (a.end_tile == 0) return VORTA_OK;
  if (p->d.head_dim == 64)
    hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(a.end_tile), dim3(64), 0, (hipStream_t)stream, a);
  else
    hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(a.end_tile), dim3(64), 0, (hipStream_t)stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(VORTA_EHIP, "launch of attn_f32_kernel: %s", hipGetErrorString(e));
  return VORTA_OK;
}

}  // namespace vorta
