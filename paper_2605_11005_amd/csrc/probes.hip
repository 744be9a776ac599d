// Measured ceilings for the benchmark: an MFMA-only loop (no memory traffic) and a plain
// device copy.  They give the rates this chip sustains under its own power management, next
// to which the kernels' figures are reported; they are not part of the expert-layer path.
#include "common.h"
#include "kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// 4 wavefronts per CU, 16 independent 32x32 accumulators each: the MFMA pipe is always busy.
__global__ __launch_bounds__(256, 1) void mfma_peak(float* sink, int iters, int random_operands) {
  f32x16 acc[16];
  for (int i = 0; i < 16; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  union { bf16x8 v; uint32_t u[4]; } a[4], b[4];
  for (int q = 0; q < 4; ++q)
    for (int j = 0; j < 4; ++j) {
      if (random_operands) {   // random sign and mantissa, magnitudes in [0.5, 2): worst-case toggling
        uint32_t h = mix32(threadIdx.x * 131u + q * 17u + j + blockIdx.x * 7919u), g = mix32(h + 12345u);
        a[q].u[j] = (h & 0x80FF80FFu) | 0x3F003F00u;
        b[q].u[j] = (g & 0x80FF80FFu) | 0x3F003F00u;
      } else {
        a[q].u[j] = 0x3F803F80u;
        b[q].u[j] = 0x3F003F00u;
      }
    }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i >> 2].v, b[i & 3].v, acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_peak(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

int launch_probe_mfma(float* sink, int iters, int random_operands, hipStream_t s) {
  hipLaunchKernelGGL(mfma_peak, dim3(device_cu_count()), dim3(256), 0, s, sink, iters, random_operands);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return MOE_OK;
  hipLaunchKernelGGL(copy_peak, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const u32x4*)src, (u32x4*)dst, n);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}
