// Measured ceilings for the benchmark: an MFMA-only loop (no memory traffic) and a plain
// device copy.  They give the rates this chip sustains under its own power management, next
// to which the kernels' figures are reported; they are not part of the expert-layer path.
#include "common.h"
#include "kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

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

// The same loop with the operands of every k-step re-read from LDS at the rate a 256 x 256 block tile with
// 128 x 128 per wavefront needs (8 fragments of 16 bytes per lane per 16 MFMAs): FEED 1 reads them with
// 16-byte reads, FEED 2 with pairs of 8-byte transposing reads.  64 KB of random bf16 pairs in LDS; the
// addresses rotate through it and stay inside it.
template <int FEED>
__global__ __launch_bounds__(256, 1) void mfma_fed(float* sink, int iters) {
  __shared__ __align__(16) uint32_t lds[16384];
  for (int i = threadIdx.x; i < 16384; i += 256) lds[i] = (mix32(i * 2654435761u + blockIdx.x) & 0x80FF80FFu) | 0x3F003F00u;
  __syncthreads();
  f32x16 acc[16];
  for (int i = 0; i < 16; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const char* base = reinterpret_cast<const char*>(lds);
  bf16x8 a[4], b[4];
  for (int it = 0; it < iters; ++it) {
    const int o = ((it & 3) * 16384 + wave * 64) & 65535;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (FEED == 1) {
        a[q] = *reinterpret_cast<const bf16x8*>(base + ((o + q * 2048 + lane * 16) & 65535));
        b[q] = *reinterpret_cast<const bf16x8*>(base + ((o + 8192 + q * 2048 + lane * 16) & 65535));
      } else {
        auto tr = [&](int off) {
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base + ((off + lane * 8) & 65535)));
          s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base + ((off + 1024 + lane * 8) & 65535)));
          return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        };
        a[q] = tr(o + q * 2048);
        b[q] = tr(o + 8192 + q * 2048);
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i >> 2], b[i & 3], acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Streaming kernels with the row movers' access width (16 bytes per thread, nontemporal): WRITES = -1 reads
// only, 0 fills, n >= 1 reads one vector and writes it n times (dst holds n regions of the source's size).
template <int WRITES>
__global__ __launch_bounds__(256) void stream_peak(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n, uint32_t* sink) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  if (WRITES == 0) {
    const u32x4 v = {1u, 2u, 3u, (uint32_t)i};
    __builtin_nontemporal_store(v, dst + i);
  } else {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    if (WRITES < 0) {
      if (v.x == 0x12345678u && v.y == 77u && v.z == 0x9abcdef0u) sink[0] = v.w;    // keeps the load alive
    } else {
#pragma unroll
      for (int w = 0; w < WRITES; ++w) __builtin_nontemporal_store(v, dst + (size_t)w * n + i);
    }
  }
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

int launch_probe_mfma_fed(float* sink, int iters, int feed, hipStream_t s) {
  if (feed == 1) hipLaunchKernelGGL(mfma_fed<1>, dim3(device_cu_count()), dim3(256), 0, s, sink, iters);
  else hipLaunchKernelGGL(mfma_fed<2>, dim3(device_cu_count()), dim3(256), 0, s, sink, iters);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_probe_stream(const void* src, void* dst, size_t bytes, int writes, uint32_t* sink, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return MOE_OK;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  const u32x4* a = (const u32x4*)src;
  u32x4* b = (u32x4*)dst;
  switch (writes) {
    case -1: hipLaunchKernelGGL(stream_peak<-1>, grid, block, 0, s, a, b, n, sink); break;
    case 0: hipLaunchKernelGGL(stream_peak<0>, grid, block, 0, s, a, b, n, sink); break;
    case 1: hipLaunchKernelGGL(stream_peak<1>, grid, block, 0, s, a, b, n, sink); break;
    case 2: hipLaunchKernelGGL(stream_peak<2>, grid, block, 0, s, a, b, n, sink); break;
    default: hipLaunchKernelGGL(stream_peak<3>, grid, block, 0, s, a, b, n, sink); break;
  }
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
