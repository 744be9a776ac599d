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

// ---- quarter-wavefront variant: 16 lanes per token (E <= 256, k <= 16) -------------------
// Four tokens per wavefront; lane s of a token's group holds the logits of experts 4s + 64i + j
// (16-byte loads).  All reductions stay inside a row of 16 lanes and use DPP row operations
// (quad permutes, half-row mirror, row mirror), which cost no LDS-crossbar traffic.  Selection
// compares (order-preserving image of the logit, then lower expert id), so ties resolve as in
// the whole-wavefront kernel and the indices are identical.
__device__ __forceinline__ int dpp_xor1(int v) { return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, true); }    // quad_perm [1,0,3,2]
__device__ __forceinline__ int dpp_xor2(int v) { return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, true); }    // quad_perm [2,3,0,1]
__device__ __forceinline__ int dpp_half_mirror(int v) { return __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, true); }
__device__ __forceinline__ int dpp_mirror(int v) { return __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, true); }

template <typename F>
__device__ __forceinline__ float row16_reduce(float v, F op) {
  v = op(v, __int_as_float(dpp_xor1(__float_as_int(v))));
  v = op(v, __int_as_float(dpp_xor2(__float_as_int(v))));
  v = op(v, __int_as_float(dpp_half_mirror(__float_as_int(v))));
  v = op(v, __int_as_float(dpp_mirror(__float_as_int(v))));
  return v;
}
// best (key, expert) of the row: larger key first, lower expert id on equal keys
__device__ __forceinline__ void row16_best(uint32_t& key, int& e) {
#define ROUTE_STEP(FN)                                              \
  {                                                                 \
    const uint32_t k2 = (uint32_t)FN((int)key);                     \
    const int e2 = FN(e);                                           \
    const bool take = k2 > key || (k2 == key && e2 < e);            \
    key = take ? k2 : key;                                          \
    e = take ? e2 : e;                                              \
  }
  ROUTE_STEP(dpp_xor1) ROUTE_STEP(dpp_xor2) ROUTE_STEP(dpp_half_mirror) ROUTE_STEP(dpp_mirror)
#undef ROUTE_STEP
}
__device__ __forceinline__ float from_ordered_bits(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}

template <int NV>   // NV = number of 4-expert vectors per lane = ceil(E / 64)
__global__ __launch_bounds__(256) void route_kernel_q(const float* __restrict__ logits, int T, int E, int k, int mode,
                                                      int e_lo, int e_cnt, int32_t* __restrict__ topk_idx,
                                                      float* __restrict__ topk_w, int32_t* __restrict__ counts) {
  extern __shared__ int32_t hist[];
  for (int i = threadIdx.x; i < e_cnt; i += blockDim.x) hist[i] = 0;
  __syncthreads();
  const int s = threadIdx.x & 15;
  const int group = threadIdx.x >> 4;                    // 16 tokens per block
  const int groups = blockDim.x >> 4;
  const int n_iter = (T + gridDim.x * groups - 1) / (gridDim.x * groups);   // same trip count for every lane (DPP needs full rows)
  for (int it = 0; it < n_iter; ++it) {
    const int t = (it * gridDim.x + blockIdx.x) * groups + group;
    const bool live = t < T;
    const float* row = logits + (size_t)(live ? t : 0) * E;
    uint32_t key[NV][4];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int e0 = 4 * s + 64 * i;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e0 < E) v = *reinterpret_cast<const float4*>(row + e0);      // E % 4 == 0
      key[i][0] = e0 < E ? ordered_bits(v.x) : 0u;
      key[i][1] = e0 < E ? ordered_bits(v.y) : 0u;
      key[i][2] = e0 < E ? ordered_bits(v.z) : 0u;
      key[i][3] = e0 < E ? ordered_bits(v.w) : 0u;
    }
    float full_max = 0.f, full_den = 1.f;
    if (mode == MOE_GATE_SOFTMAX) {
      float m = -INFINITY;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (4 * s + 64 * i < E) m = fmaxf(m, from_ordered_bits(key[i][j]));
      full_max = row16_reduce(m, [](float a, float b) { return fmaxf(a, b); });
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (4 * s + 64 * i < E) acc += __expf(from_ordered_bits(key[i][j]) - full_max);
      full_den = row16_reduce(acc, [](float a, float b) { return a + b; });
    }
    float my_logit = 0.f;
    int my_idx = -1;
    for (int r = 0; r < k; ++r) {
      uint32_t bk = 0u;
      int be = 0x7FFFFFFF;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (key[i][j] > bk) { bk = key[i][j]; be = 4 * s + 64 * i + j; }   // ascending ids: first of equals wins
      row16_best(bk, be);
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (be == 4 * s + 64 * i + j) key[i][j] = 0u;                       // taken (real keys are never 0)
      if (s == r) { my_logit = from_ordered_bits(bk); my_idx = be; }
    }
    const bool act = s < k;
    float w;
    if (mode == MOE_GATE_SIGMOID_RENORM) {
      const float sg = act ? 1.0f / (1.0f + __expf(-my_logit)) : 0.f;
      w = sg / row16_reduce(sg, [](float a, float b) { return a + b; });
    } else if (mode == MOE_GATE_SOFTMAX_RENORM) {
      const float top = row16_reduce(act ? my_logit : -INFINITY, [](float a, float b) { return fmaxf(a, b); });
      const float ex = act ? __expf(my_logit - top) : 0.f;
      w = ex / row16_reduce(ex, [](float a, float b) { return a + b; });
    } else {
      w = __expf(my_logit - full_max) / full_den;
    }
    if (act && live) {
      topk_idx[(size_t)t * k + s] = my_idx;
      topk_w[(size_t)t * k + s] = w;
      const int le = my_idx - e_lo;
      if (le >= 0 && le < e_cnt) atomicAdd(&hist[le], 1);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < e_cnt; i += blockDim.x) {
    const int c = hist[i];
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
  size_t shm_q = (size_t)(e_cnt > 0 ? e_cnt : 1) * sizeof(int32_t);
  if (E <= 256 && k <= 16 && E % 4 == 0 && ((uintptr_t)logits & 15) == 0) {
    // 16 lanes per token
    int qb = (T + 15) / 16;
    const int qmax = device_cu_count() * 8;
    if (qb > qmax) qb = qmax;
    const int nv = (E + 63) / 64;
#define ROUTE_Q(V)                                                                                     \
  hipLaunchKernelGGL(route_kernel_q<V>, dim3(qb), dim3(256), shm_q, s, logits, T, E, k, gate_mode, e_lo, \
                     e_cnt, topk_idx, topk_w, counts)
    if (nv <= 1) ROUTE_Q(1);
    else if (nv <= 2) ROUTE_Q(2);
    else ROUTE_Q(4);
#undef ROUTE_Q
    HIP_CHECK_LAUNCH();
    return MOE_OK;
  }
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
