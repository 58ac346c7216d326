// fp32 routed attention for gfx950: the exact-precision path (small layers, 1e-5 parity).
// Inputs and outputs are fp32; everything in between is fp64, so the result is the correctly
// computed softmax(scale Q K^T) V rounded once to fp32, whatever the number of keys: a product
// of two fp32 values is exact in fp64, and the sums (head_dim terms per score, all keys per
// output element) carry fp64 rounding only.  (An all-fp32 version of this kernel drifted past
// 1e-5 from about three thousand keys on: sequential fp32 accumulation over the key stream.)
//
// A workgroup of four wavefronts owns 64 query rows; four neighbouring lanes share a row, lane
// quarter c owning the 16-byte chunks e with e % 4 == c of the query row and of the output
// accumulator (neighbouring chunks, so the four reads of a K or V row hit different LDS banks
// while the 16 rows of a wavefront read the same addresses: LDS broadcasts).  Keys stream
// through LDS 32 rows at a time; a score is the sum over the quad of four partial dot products.
// Online softmax in fp64 with the running maximum.  Throughput is not a goal of this kernel;
// the bf16 MFMA kernel is the fast path.
#include <hip/hip_runtime.h>

#include "vorta_attn_common.h"

namespace vorta {

template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnArgs a) {
  constexpr int BM = 64, BN = 32;
  constexpr int CH = D / 16;                 // 16-byte chunks of a row per lane
  __shared__ float sK[BN][D];
  __shared__ float sV[BN][D];
  const WorkItem w = decode_item<BM, D>(a, blockIdx.x);
  const float* Q = (const float*)(w.seg == 0 ? a.q0 : w.seg == 1 ? a.qc : a.qt) + w.q_off;
  const float* K = (const float*)(w.seg == 0 ? a.k0 : w.seg == 1 ? a.kc : a.kt) + w.kv_off;
  const float* V = (const float*)(w.seg == 0 ? a.v0 : w.seg == 1 ? a.vc : a.vt) + w.kv_off;
  float* O = (float*)(w.seg == 0 ? a.o0 : w.seg == 1 ? a.oc : a.ot) + w.o_off;
  if (w.n_rows <= 0) return;       // q-block past the end of a clipped tile
  const int t = threadIdx.x;
  const int quarter = t & 3, r_local = t >> 2;
  const long my_row = w.row(min(r_local, w.n_rows - 1));

  float4 q[CH];
  double o[CH][4];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    q[i] = ((const float4*)(Q + my_row * w.row_stride))[4 * i + quarter];
    o[i][0] = o[i][1] = o[i][2] = o[i][3] = 0.0;
  }
  double m = -INFINITY, l = 0.0;
  const double scale = (double)a.scale;

  for (int r = 0; r < w.n_runs; ++r) {
    const int start = w.runs ? w.runs[2 * r] : 0;
    const int len = w.runs ? w.runs[2 * r + 1] : w.single_len;
    for (int pos = 0; pos < len; pos += BN) {
      const int n_valid = min(BN, len - pos);
      __syncthreads();
      for (int c = t; c < BN * D / 4; c += 256) {
        const int j = c / (D / 4), e = c - j * (D / 4);
        const long row = start + pos + min(j, n_valid - 1);   // rows past the run repeat its last row
        ((float4*)&sK[j][0])[e] = ((const float4*)(K + row * w.row_stride))[e];
        ((float4*)&sV[j][0])[e] = ((const float4*)(V + row * w.row_stride))[e];
      }
      __syncthreads();
      double s[BN];
      double mt = -INFINITY;
#pragma unroll
      for (int j = 0; j < BN; ++j) {
        double dot = 0.0;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          const float4 kk = ((const float4*)&sK[j][0])[4 * i + quarter];
          dot = fma((double)q[i].x, (double)kk.x, dot);
          dot = fma((double)q[i].y, (double)kk.y, dot);
          dot = fma((double)q[i].z, (double)kk.z, dot);
          dot = fma((double)q[i].w, (double)kk.w, dot);
        }
        dot += __shfl_xor(dot, 1, 64);
        dot += __shfl_xor(dot, 2, 64);
        s[j] = j < n_valid ? dot * scale : -INFINITY;
        mt = fmax(mt, s[j]);
      }
      const double m_new = fmax(m, mt);
      const double alpha = exp(m - m_new);   // 0 for the first block
      l *= alpha;
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        o[i][0] *= alpha; o[i][1] *= alpha; o[i][2] *= alpha; o[i][3] *= alpha;
      }
#pragma unroll
      for (int j = 0; j < BN; ++j) {
        const double pj = exp(s[j] - m_new);
        l += pj;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          const float4 vv = ((const float4*)&sV[j][0])[4 * i + quarter];
          o[i][0] = fma(pj, (double)vv.x, o[i][0]);
          o[i][1] = fma(pj, (double)vv.y, o[i][1]);
          o[i][2] = fma(pj, (double)vv.z, o[i][2]);
          o[i][3] = fma(pj, (double)vv.w, o[i][3]);
        }
      }
      m = m_new;
    }
  }
  if (r_local < w.n_rows) {
    const double inv = 1.0 / l;
    float4* dst = (float4*)(O + my_row * w.row_stride);
#pragma unroll
    for (int i = 0; i < CH; ++i)
      dst[4 * i + quarter] = make_float4((float)(o[i][0] * inv), (float)(o[i][1] * inv), (float)(o[i][2] * inv),
                                         (float)(o[i][3] * inv));
  }
}

int launch_attention_f32(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream) {
  AttnArgs a;
  if (int rc = fill_attn_args(p, rl, io, 64, WIN_ALL, &a)) return rc;
  if (a.end_tile == 0) return VORTA_OK;
  if (p->d.head_dim == 64)
    hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(a.end_tile), dim3(256), 0, (hipStream_t)stream, a);
  else
    hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(a.end_tile), dim3(256), 0, (hipStream_t)stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(VORTA_EHIP, "launch of attn_f32_kernel: %s", hipGetErrorString(e));
  return VORTA_OK;
}

}  // namespace vorta
