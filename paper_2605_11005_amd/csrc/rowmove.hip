// Row movers: dispatch (token order -> expert order) and combine (expert order -> token
// order, gate-weighted).  Both are token-major with one wavefront per token, so every row
// of x / o is read exactly once and every row of xp / y is written exactly once:
//   dispatch : read x[t] once (skipped when the token has no local slot), write it to each
//              of the token's local rows            -> (U + R) * d * b bytes
//   combine  : read the token's local rows, write y[t] once (zeros when none)
//                                                   -> (R + T) * d * b bytes
// Accesses are 16 bytes per lane, whole rows per wavefront, several loads in flight.
#include "common.h"
#include "kernels.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int WPB = 4;   // wavefronts (tokens) per block

template <bool BF16>
__device__ __forceinline__ u32x4 scale_vec(u32x4 v, float sc) {
  if (BF16) {
    u32x4 r;
    r.x = pack_bf16x2(bf16lo(v.x) * sc, bf16hi(v.x) * sc);
    r.y = pack_bf16x2(bf16lo(v.y) * sc, bf16hi(v.y) * sc);
    r.z = pack_bf16x2(bf16lo(v.z) * sc, bf16hi(v.z) * sc);
    r.w = pack_bf16x2(bf16lo(v.w) * sc, bf16hi(v.w) * sc);
    return r;
  } else {
    u32x4 r;
    r.x = __float_as_uint(__uint_as_float(v.x) * sc);
    r.y = __float_as_uint(__uint_as_float(v.y) * sc);
    r.z = __float_as_uint(__uint_as_float(v.z) * sc);
    r.w = __float_as_uint(__uint_as_float(v.w) * sc);
    return r;
  }
}

// row_vecs = number of 16-byte vectors per row
template <bool BF16, bool SCALED>
__global__ __launch_bounds__(WPB * WAVE) void dispatch_rows(const u32x4* __restrict__ x, int T, int row_vecs, int k,
                                                           const int32_t* __restrict__ inv,
                                                           const float* __restrict__ row_scale,
                                                           u32x4* __restrict__ xp) {
  const int lane = lane_id();
  const int t = blockIdx.x * WPB + threadIdx.x / WAVE;
  if (t >= T) return;
  int my_row = -1;
  float my_sc = 1.0f;
  if (lane < k) {
    my_row = inv[(size_t)t * k + lane];
    if (SCALED) my_sc = row_scale[(size_t)t * k + lane];
  }
  unsigned long long local = __ballot(my_row >= 0);
  if (!local) return;
  const u32x4* src = x + (size_t)t * row_vecs;
  for (int c0 = 0; c0 < row_vecs; c0 += 4 * WAVE) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int c = c0 + u * WAVE + lane;
      if (c < row_vecs) v[u] = __builtin_nontemporal_load(src + c);
    }
    unsigned long long m = local;
    while (m) {
      const int j = __ffsll((long long)m) - 1;
      m &= m - 1;
      const int row = __shfl(my_row, j, WAVE);
      const float sc = SCALED ? __shfl(my_sc, j, WAVE) : 1.0f;
      u32x4* dst = xp + (size_t)row * row_vecs;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int c = c0 + u * WAVE + lane;
        if (c < row_vecs) {
          u32x4 o = SCALED ? scale_vec<BF16>(v[u], sc) : v[u];
          __builtin_nontemporal_store(o, dst + c);
        }
      }
    }
  }
}

template <bool BF16>
__device__ __forceinline__ void fma_vec(float* acc, u32x4 v, float w) {
  if (BF16) {
    acc[0] += w * bf16lo(v.x); acc[1] += w * bf16hi(v.x);
    acc[2] += w * bf16lo(v.y); acc[3] += w * bf16hi(v.y);
    acc[4] += w * bf16lo(v.z); acc[5] += w * bf16hi(v.z);
    acc[6] += w * bf16lo(v.w); acc[7] += w * bf16hi(v.w);
  } else {
    acc[0] += w * __uint_as_float(v.x); acc[1] += w * __uint_as_float(v.y);
    acc[2] += w * __uint_as_float(v.z); acc[3] += w * __uint_as_float(v.w);
  }
}

template <bool BF16>
__device__ __forceinline__ u32x4 pack_acc(const float* acc) {
  u32x4 r;
  if (BF16) {
    r.x = pack_bf16x2(acc[0], acc[1]); r.y = pack_bf16x2(acc[2], acc[3]);
    r.z = pack_bf16x2(acc[4], acc[5]); r.w = pack_bf16x2(acc[6], acc[7]);
  } else {
    r.x = __float_as_uint(acc[0]); r.y = __float_as_uint(acc[1]);
    r.z = __float_as_uint(acc[2]); r.w = __float_as_uint(acc[3]);
  }
  return r;
}

template <bool BF16>
__global__ __launch_bounds__(WPB * WAVE) void combine_rows(const u32x4* __restrict__ o, int T, int row_vecs, int k,
                                                          const int32_t* __restrict__ inv,
                                                          const float* __restrict__ topk_w,
                                                          u32x4* __restrict__ y) {
  const int lane = lane_id();
  const int t = blockIdx.x * WPB + threadIdx.x / WAVE;
  if (t >= T) return;
  int my_row = -1;
  float my_w = 1.0f;
  if (lane < k) {
    my_row = inv[(size_t)t * k + lane];
    if (topk_w) my_w = topk_w[(size_t)t * k + lane];
  }
  const unsigned long long local = __ballot(my_row >= 0);
  u32x4* dst = y + (size_t)t * row_vecs;
  for (int c0 = 0; c0 < row_vecs; c0 += 2 * WAVE) {
    float acc[2][8];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[u][i] = 0.f;
    unsigned long long m = local;
    while (m) {                                       // ascending slot j
      const int j = __ffsll((long long)m) - 1;
      m &= m - 1;
      const int row = __shfl(my_row, j, WAVE);
      const float w = __shfl(my_w, j, WAVE);
      const u32x4* src = o + (size_t)row * row_vecs;
      u32x4 v[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int c = c0 + u * WAVE + lane;
        if (c < row_vecs) v[u] = __builtin_nontemporal_load(src + c);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int c = c0 + u * WAVE + lane;
        if (c < row_vecs) fma_vec<BF16>(acc[u], v[u], w);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      int c = c0 + u * WAVE + lane;
      if (c < row_vecs) __builtin_nontemporal_store(pack_acc<BF16>(acc[u]), dst + c);
    }
  }
}

}  // namespace

int launch_dispatch_rows(const void* x, int dtype, int T, int d, int k, const int32_t* inv,
                         const float* row_scale, void* xp, hipStream_t s) {
  if (T == 0) return MOE_OK;
  ProfScope prof(MOE_K_DISPATCH, s);
  const int row_vecs = dtype == MOE_BF16 ? d / 8 : d / 4;
  dim3 grid((T + WPB - 1) / WPB), block(WPB * WAVE);
  const u32x4* xs = (const u32x4*)x;
  u32x4* xd = (u32x4*)xp;
  if (dtype == MOE_BF16) {
    if (row_scale) hipLaunchKernelGGL((dispatch_rows<true, true>), grid, block, 0, s, xs, T, row_vecs, k, inv, row_scale, xd);
    else hipLaunchKernelGGL((dispatch_rows<true, false>), grid, block, 0, s, xs, T, row_vecs, k, inv, row_scale, xd);
  } else {
    if (row_scale) hipLaunchKernelGGL((dispatch_rows<false, true>), grid, block, 0, s, xs, T, row_vecs, k, inv, row_scale, xd);
    else hipLaunchKernelGGL((dispatch_rows<false, false>), grid, block, 0, s, xs, T, row_vecs, k, inv, row_scale, xd);
  }
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_combine_rows(const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                        const float* topk_w, void* y, hipStream_t s) {
  if (T == 0) return MOE_OK;
  ProfScope prof(MOE_K_COMBINE, s);
  const int row_vecs = dtype == MOE_BF16 ? d / 8 : d / 4;
  dim3 grid((T + WPB - 1) / WPB), block(WPB * WAVE);
  if (dtype == MOE_BF16)
    hipLaunchKernelGGL((combine_rows<true>), grid, block, 0, s, (const u32x4*)o, T, row_vecs, k, inv, topk_w, (u32x4*)y);
  else
    hipLaunchKernelGGL((combine_rows<false>), grid, block, 0, s, (const u32x4*)o, T, row_vecs, k, inv, topk_w, (u32x4*)y);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}
