// Measurement aid, built into a library of its own (libvorta_probe.so) that only the benchmark
// loads; not part of the attention path or of libvorta's ABI: the matrix-pipe rate this chip
// sustains for a bf16 matrix instruction when little or nothing else runs, as a function of the
// operand data, of the instruction's shape and of the number of plain vector instructions issued
// next to it.  The nominal peak (256 CUs x 4 SIMDs x 1024 FLOPs per cycle x 2.4 GHz) assumes the
// nominal clock; under sustained matrix load the clock is set by power, and the power of a
// matrix instruction depends on how many operand bits toggle and on its shape
// (v_mfma_f32_16x16x32_bf16 updates half as many accumulator elements per FLOP as
// v_mfma_f32_32x32x16_bf16 and sustains a higher rate on the same random data).  On zero operands
// nothing toggles and the rate shows the issue limits instead: a matrix instruction of either
// shape keeps a SIMD's vector issue port for 8 cycles, which is a quarter of the 32x32x16's
// time on the matrix pipe but half of the 16x16x32's.  The attention kernels are priced against
// the nominal peak; this probe says how much of it data like theirs can reach at all.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace vorta {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// 8 wavefronts per workgroup (two per SIMD), one workgroup per CU (the launch asks for more than
// half a CU's LDS); every wavefront loops over 8 operand pairs held in registers and 4 independent
// accumulators.
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


// The same with a choice of shape and with vector instructions in between: independent
// accumulators (4 of 32x32, SHAPE 32, or 8 of 16x16, SHAPE 16: the same FLOPs per trip) and KV
// independent v_fma_f32 per 16 cycles of matrix-pipe time behind each matrix instruction.  (The
// plain 32x32x16 stream keeps the kernel above: compiled from this template with KV = 0 the same
// instruction sequence, with its four accumulators numbered in the opposite order, ran a quarter
// slower on every box tried -- explicit-register replicas of both loops did not differ, so the
// cause is not known; the other instances are not affected, by their rates on zero operands.)
template <int SHAPE, int KV>
__global__ __launch_bounds__(512, 1) void mfma_mix_kernel(const uint4* __restrict__ operands, int iters,
                                                           float* __restrict__ sink, long long* __restrict__ clocks) {
  constexpr int NACC = SHAPE == 32 ? 4 : 8, PER = SHAPE == 32 ? 2 * KV : KV;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, operands[(i * 2) * 64 + (threadIdx.x & 63)]);
    b[i] = __builtin_bit_cast(bf16x8, operands[(i * 2 + 1) * 64 + (threadIdx.x & 63)]);
  }
  f32x16 c32[4];
  f32x4 c16[8];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) c32[j][v] = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) c16[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  float x[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) x[k] = 1e-3f * (float)threadIdx.x + (float)k;
  const long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int j = 0; j < NACC; ++j) {
        if constexpr (KV > 0) __builtin_amdgcn_sched_barrier(0);
        if constexpr (SHAPE == 32)
          c32[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + j) & 7], b[(i + 2 * j) & 7], c32[j], 0, 0, 0);
        else
          c16[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(i + j) & 7], b[(i + 2 * j) & 7], c16[j], 0, 0, 0);
#pragma unroll
        for (int k = 0; k < PER; ++k) x[(j * PER + k) & 7] = __builtin_fmaf(x[(j * PER + k) & 7], 0.999f, 1e-3f);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = __builtin_amdgcn_s_memtime() - t0;          // shader clock ticks
    clocks[1] = __builtin_amdgcn_s_memrealtime() - r0;      // 100 MHz ticks
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) s += c32[j][0] + c32[j][15];
#pragma unroll
  for (int j = 0; j < 8; ++j) s += c16[j][0] + c16[j][3] + x[j];
  sink[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace vorta

// Runs one bf16 matrix instruction shape (shape 32: v_mfma_f32_32x32x16_bf16, 16:
// v_mfma_f32_16x16x32_bf16; 8 wavefronts per workgroup, `workgroups` workgroups, `iters` trips of
// 2^20 FLOPs per wavefront) on the operand bits the caller supplies, with vector_ops (0, 2, 3
// or 4) independent v_fma_f32 per 16 cycles of matrix-pipe time issued behind every matrix
// instruction.  operands: device, 16 x 64 x 16 bytes (8 A and 8 B fragments per lane); sink:
// device float[workgroups * 512]; clocks: device int64[2], receives shader-clock ticks and
// 100 MHz ticks of workgroup 0.  FLOPs = workgroups * 8 * iters * 2^20.  Returns 0, -1 (bad
// argument) or the hipError_t of the launch.
extern "C" int mfma_probe_rate(const void* operands, int32_t iters, int32_t workgroups, int32_t shape,
                               int32_t vector_ops, void* sink, void* clocks, void* stream) {
  using namespace vorta;
  if (!operands || !sink || !clocks || iters < 1 || workgroups < 1) return -1;
  typedef void (*kernel_t)(const uint4*, int, float*, long long*);
  kernel_t k = nullptr;
  if (shape == 32)
    k = vector_ops == 0 ? mfma_rate_kernel : vector_ops == 2 ? mfma_mix_kernel<32, 2>
      : vector_ops == 3 ? mfma_mix_kernel<32, 3> : vector_ops == 4 ? mfma_mix_kernel<32, 4> : nullptr;
  else if (shape == 16)
    k = vector_ops == 0 ? mfma_mix_kernel<16, 0> : vector_ops == 2 ? mfma_mix_kernel<16, 2>
      : vector_ops == 3 ? mfma_mix_kernel<16, 3> : vector_ops == 4 ? mfma_mix_kernel<16, 4> : nullptr;
  if (!k) return -1;
  // 96 KB of (unused) LDS per workgroup: one workgroup, two wavefronts per SIMD, on every CU for
  // every instance, however few registers it needs -- the attention kernels' occupancy
  constexpr int kLds = 96 * 1024;
  hipError_t e = hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (e != hipSuccess) return (int)e;
  hipLaunchKernelGGL(k, dim3(workgroups), dim3(512), kLds, (hipStream_t)stream, (const uint4*)operands, iters,
                     (float*)sink, (long long*)clocks);
  return (int)hipGetLastError();
}
