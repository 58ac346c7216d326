// Measurement aid, built into a library of its own (libvorta_probe.so) that only the benchmark
// loads; not part of the attention path or of libvorta's ABI: the matrix-pipe rate this chip sustains for
// v_mfma_f32_32x32x16_bf16 when nothing else runs, as a function of the operand data.  The
// nominal peak (256 CUs x 4 SIMDs x one 32x32x16 instruction per 32 cycles x 2.4 GHz) assumes
// the nominal clock; under sustained matrix load the clock is set by power, and the power of a
// matrix instruction depends on how many operand bits toggle.  The attention kernels are priced
// against the nominal peak; this probe says how much of it random bf16 data can reach at all.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace vorta {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// 8 wavefronts per workgroup (two per SIMD), one workgroup per CU-slot; every wavefront loops
// over 8 operand pairs held in registers and 4 independent accumulators.
__global__ __launch_bounds__(512, 1) void mfma_rate_kernel(const uint4* __restrict__ operands, int iters,
                                                           float* __restrict__ sink, long long* __restrict__ clocks) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, operands[(i * 2) * 64 + (threadIdx.x & 63)]);
    b[i] = __builtin_bit_cast(bf16x8, operands[(i * 2 + 1) * 64 + (threadIdx.x & 63)]);
  }
  f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[j][v] = 0.f;
  const long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + j) & 7], b[(i + 2 * j) & 7], c[j], 0, 0, 0);
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = __builtin_amdgcn_s_memtime() - t0;          // shader clock ticks
    clocks[1] = __builtin_amdgcn_s_memrealtime() - r0;      // 100 MHz ticks
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) s += c[j][0] + c[j][15];
  sink[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace vorta

// Runs only v_mfma_f32_32x32x16_bf16 (8 wavefronts per workgroup, `workgroups` workgroups,
// `iters` x 32 instructions per wavefront) on the operand bits the caller supplies.  operands:
// device, 16 x 64 x 16 bytes (8 A and 8 B fragments per lane); sink: device float[workgroups * 512];
// clocks: device int64[2], receives shader-clock ticks and 100 MHz ticks of workgroup 0.
// FLOPs = workgroups * 8 * iters * 32 * 32768.  Returns 0, -1 (bad argument) or the hipError_t
// of the launch.
extern "C" int mfma_probe_rate(const void* operands, int32_t iters, int32_t workgroups, void* sink, void* clocks,
                               void* stream) {
  using namespace vorta;
  if (!operands || !sink || !clocks || iters < 1 || workgroups < 1) return -1;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, (const uint4*)operands,
                     iters, (float*)sink, (long long*)clocks);
  return (int)hipGetLastError();
}
