// Shared device helpers for the gfx950 MoE kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define WAVE 64

typedef uint16_t bf16_t;   // raw bfloat16 bits in memory

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even; inputs are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two floats -> packed bf16 pair, round-to-nearest-even, in one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float bf16lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16hi(uint32_t v) { return __uint_as_float(v & 0xFFFF0000u); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }

// logistic function with the hardware exp2 and reciprocal (about 1 ulp each; used by the bf16
// epilogues, whose results are rounded to 8 bits of mantissa)
__device__ __forceinline__ float sigmoid_fast(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896f * z));
}
__device__ __forceinline__ float silu_f(float z) { return z * sigmoid_fast(z); }
// returns silu(z) and writes silu'(z) = s (1 + z (1 - s))
__device__ __forceinline__ float silu_grad_f(float z, float* ds) {
  float s = sigmoid_fast(z);
  *ds = s * (1.0f + z * (1.0f - s));
  return z * s;
}

#define HIP_CHECK_LAUNCH()                                  \
  do {                                                      \
    if (hipGetLastError() != hipSuccess) return MOE_EHIP;   \
  } while (0)
