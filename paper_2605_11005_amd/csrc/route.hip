// Top-k gating: one wavefront per token.
//
// Each lane holds ceil(E/64) logits of the token's row (coalesced loads).  Selection runs
// k rounds of a wave-wide arg-max on a 64-bit key = (order-preserving image of the fp32
// logit, ~expert id), so that equal logits resolve to the lower expert id and the result
// does not depend on any exp() implementation.  Lane j keeps the j-th winner; the gate
// weights are then formed from the k kept logits with wave reductions.  Local-expert
// counts go through an LDS histogram per block and one integer atomic per (block, expert):
// integer addition commutes, so the counts are reproducible.
#include "common.h"
#include "kernels.h"

namespace {

__device__ __forceinline__ uint32_t ordered_bits(float v) {
  uint32_t u = __float_as_uint(v + 0.0f);       // -0 -> +0: the two zeros must tie
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    unsigned long long o = __shfl_xor(v, off, WAVE);
    v = o > v ? o : v;
  }
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, WAVE));
  return v;
}

__global__ void zero_i32(int32_t* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

template <int VPL>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                    int mode, int e_lo, int e_cnt,
                                                    int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w,
                                                    int32_t* __restrict__ counts) {
  extern __shared__ int32_t hist[];
  for (int i = threadIdx.x; i < e_cnt; i += blockDim.x) hist[i] = 0;
  __syncthreads();

  const int lane = lane_id();
  const int wave = threadIdx.x / WAVE;
  const int waves_per_block = blockDim.x / WAVE;
  for (int t = blockIdx.x * waves_per_block + wave; t < T; t += gridDim.x * waves_per_block) {
    const float* row = logits + (size_t)t * E;
    float v[VPL];
    unsigned long long key[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      int e = lane + i * WAVE;
      v[i] = e < E ? row[e] : 0.0f;
      key[i] = e < E ? (((unsigned long long)ordered_bits(v[i]) << 32) | (uint32_t)(~(uint32_t)e)) : 0ull;
    }
    float full_max = 0.f, full_den = 1.f;
    if (mode == MOE_GATE_SOFTMAX) {
      float m = -INFINITY;
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (lane + i * WAVE < E) m = fmaxf(m, v[i]);
      full_max = wave_max(m);
      float sacc = 0.f;
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (lane + i * WAVE < E) sacc += __expf(v[i] - full_max);
      full_den = wave_sum(sacc);
    }

    float my_logit = 0.f;   // lane j < k: logit of the j-th best expert
    int my_idx = -1;
    for (int j = 0; j < k; ++j) {
      unsigned long long best = key[0];
#pragma unroll
      for (int i = 1; i < VPL; ++i) best = key[i] > best ? key[i] : best;
      best = wave_max_u64(best);
      const int e = (int)(~(uint32_t)(best & 0xFFFFFFFFull));
      const int owner = e & (WAVE - 1), slot = e >> 6;
      float won = 0.f;
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (i == slot) {
          won = v[i];
          if (lane == owner) key[i] = 0ull;
        }
      won = __shfl(won, owner, WAVE);
      if (lane == j) { my_logit = won; my_idx = e; }
    }

    const bool act = lane < k;
    float w;
    if (mode == MOE_GATE_SIGMOID_RENORM) {
      float sg = act ? 1.0f / (1.0f + __expf(-my_logit)) : 0.f;
      w = sg / wave_sum(sg);
    } else if (mode == MOE_GATE_SOFTMAX_RENORM) {
      // softmax over all E renormalised over the selection == softmax over the k kept logits
      float top = __shfl(my_logit, 0, WAVE);
      float ex = act ? __expf(my_logit - top) : 0.f;
      w = ex / wave_sum(ex);
    } else {
      w = __expf(my_logit - full_max) / full_den;
    }
    if (act) {
      topk_idx[(size_t)t * k + lane] = my_idx;
      topk_w[(size_t)t * k + lane] = w;
      int le = my_idx - e_lo;
      if (le >= 0 && le < e_cnt) atomicAdd(&hist[le], 1);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < e_cnt; i += blockDim.x) {
    int c = hist[i];
    if (c) atomicAdd(&counts[i], c);
  }
}

}  // namespace

int launch_route(const float* logits, int T, int E, int k, int gate_mode, int e_lo, int e_cnt,
                 int32_t* topk_idx, float* topk_w, int32_t* counts, hipStream_t s) {
  if (e_cnt > 0) {
    hipLaunchKernelGGL(zero_i32, dim3((e_cnt + 255) / 256), dim3(256), 0, s, counts, e_cnt);
    HIP_CHECK_LAUNCH();
  }
  if (T == 0) return MOE_OK;
  ProfScope prof(MOE_K_ROUTE, s);
  const int wpb = 4;
  int blocks = (T + wpb - 1) / wpb;
  int maxb = device_cu_count() * 8;
  if (blocks > maxb) blocks = maxb;
  size_t shm = (size_t)(e_cnt > 0 ? e_cnt : 1) * sizeof(int32_t);
  int vpl = (E + WAVE - 1) / WAVE;
#define ROUTE_CASE(V)                                                                             \
  hipLaunchKernelGGL(route_kernel<V>, dim3(blocks), dim3(256), shm, s, logits, T, E, k, gate_mode, \
                     e_lo, e_cnt, topk_idx, topk_w, counts)
  if (vpl <= 1) ROUTE_CASE(1);
  else if (vpl <= 2) ROUTE_CASE(2);
  else if (vpl <= 4) ROUTE_CASE(4);
  else if (vpl <= 8) ROUTE_CASE(8);
  else ROUTE_CASE(16);
#undef ROUTE_CASE
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}
