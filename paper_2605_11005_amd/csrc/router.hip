// The trainable gate around the expert layer: router GEMM, fused backward of combine (d_o and the
// gradient of the gate weights in one pass over dy), gradient through the gate weights to the
// logits, and the router's backward GEMMs.
//
// Large bf16 shapes (E % 64 == 0, d % 64 == 0) run on the matrix cores through the grouped-GEMM
// kernel of expert_bf16.hip; every other shape (fp32, or a handful of experts) takes the plain
// LDS-tiled FMA kernels below, which accept any size.  The contraction over the tokens (dWr) is
// always split into fixed chunks whose fp32 sums are added in ascending order, so the result
// does not depend on scheduling.
#include "common.h"
#include "kernels.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float ldf(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void stf(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}

constexpr int TM = 64, TN = 64, TK = 16;

// C[r,n] (=|+=) sum_k A[r,k] * B[k*b_rs + n*b_cs], r in [0,M), n in [0,N); fp32 accumulation in
// ascending k.  grid = (N tiles, M tiles), 256 threads, 4x4 outputs per thread.
template <typename TA, typename TB, typename TC>
__global__ __launch_bounds__(256) void gemm_rows_valu(const TA* __restrict__ A, int lda, const TB* __restrict__ B,
                                                     long b_rs, long b_cs, TC* __restrict__ C, int ldc, int M,
                                                     int N, int K, int beta) {
  const int row0 = blockIdx.y * TM, col0 = blockIdx.x * TN;
  __shared__ float sa[TK][TM + 1], sb[TK][TN + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
    for (int i = threadIdx.x; i < TM * TK; i += 256) {
      const int m = i / TK, kk = i % TK;
      const int r = row0 + m, kidx = k0 + kk;
      sa[kk][m] = (r < M && kidx < K) ? ldf(A, (size_t)r * lda + kidx) : 0.f;
    }
    for (int i = threadIdx.x; i < TN * TK; i += 256) {
      int n, kk;
      if (b_cs == 1) { n = i % TN; kk = i / TN; } else { kk = i % TK; n = i / TK; }
      const int c = col0 + n, kidx = k0 + kk;
      sb[kk][n] = (c < N && kidx < K) ? ldf(B, (size_t)kidx * b_rs + (size_t)c * b_cs) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = sa[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = sb[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = row0 + ty * 4 + i;
    if (r >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = col0 + tx * 4 + j;
      if (c < N) {
        const size_t idx = (size_t)r * ldc + c;
        stf(C, idx, beta ? ldf(C, idx) + acc[i][j] : acc[i][j]);
      }
    }
  }
}

// partial[z][i][j] = sum over rows r of chunk z of P[r,i] * Q[r,j]; chunk z = [z*chunk, min((z+1)*chunk, rows)).
// grid = (N tiles, M tiles, chunks)
template <typename TP>
__global__ __launch_bounds__(256) void gemm_tn_valu(const TP* __restrict__ P, int ldp, const float* __restrict__ Q,
                                                   int ldq, float* __restrict__ partial, int M, int N, int rows,
                                                   int chunk) {
  const long long lo_l = (long long)blockIdx.z * chunk;
  const int lo = (int)(lo_l < rows ? lo_l : rows);
  const int hi = (int)(lo_l + chunk < rows ? lo_l + chunk : rows);
  const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TN;
  __shared__ float sa[TK][TM + 1], sb[TK][TN + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int r0 = lo; r0 < hi; r0 += TK) {
    for (int t = threadIdx.x; t < TM * TK; t += 256) {
      const int m = t % TM, kk = t / TM;
      const int r = r0 + kk, i = i0 + m;
      sa[kk][m] = (r < hi && i < M) ? ldf(P, (size_t)r * ldp + i) : 0.f;
    }
    for (int t = threadIdx.x; t < TN * TK; t += 256) {
      const int n = t % TN, kk = t / TN;
      const int r = r0 + kk, j = j0 + n;
      sb[kk][n] = (r < hi && j < N) ? Q[(size_t)r * ldq + j] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = sa[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = sb[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
  float* out = partial + (size_t)blockIdx.z * M * N;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ii = i0 + ty * 4 + i;
    if (ii >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int jj = j0 + tx * 4 + j;
      if (jj < N) out[(size_t)ii * N + jj] = acc[i][j];
    }
  }
}

// out[i] = (beta ? out[i] : 0) + partial[0][i] + partial[1][i] + ...   (ascending chunk order)
template <typename TOut>
__global__ void reduce_chunks(const float* __restrict__ partial, int chunks, size_t n, TOut* __restrict__ out,
                              int beta) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float s = 0.f;
    for (int c = 0; c < chunks; ++c) s += partial[(size_t)c * n + i];
    stf(out, i, beta ? ldf(out, i) + s : s);
  }
}

// dx[t,c] (=|+=) sum_e dl[t,e] * Wr[c,e] for a small number of experts (the plain path's router term of dx):
// one thread per 4 consecutive columns c, whose 4*E weights are contiguous in memory; the token's
// dlogits row sits in LDS.  1-D grid: block = (token, group of 1024 columns), column group fastest.
template <typename TW>
__global__ __launch_bounds__(256) void router_dx_small_e(const float* __restrict__ dl, const TW* __restrict__ wr,
                                                        TW* __restrict__ dx, int d, int E, int beta, int col_groups) {
  __shared__ float row[MOE_MAX_EXPERTS];
  const int t = blockIdx.x / col_groups;
  const int cg = blockIdx.x - t * col_groups;
  for (int e = threadIdx.x; e < E; e += 256) row[e] = dl[(size_t)t * E + e];
  __syncthreads();
  const int c0 = (cg * 256 + threadIdx.x) * 4;
  if (c0 >= d) return;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (c0 + i >= d) break;
    const TW* w = wr + (size_t)(c0 + i) * E;
    float s = 0.f;
    for (int e = 0; e < E; ++e) s += row[e] * ldf(w, e);
    acc[i] = s;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (c0 + i >= d) break;
    const size_t idx = (size_t)t * d + c0 + i;
    stf(dx, idx, beta ? ldf(dx, idx) + acc[i] : acc[i]);
  }
}

// logits[t,e] = sum_c x[t,c] * Wr[c,e] for a small number of experts: one block per token, eight
// experts per pass (their weights are contiguous in a row of Wr), columns strided over the threads,
// sums reduced lanes -> wavefront -> block in a fixed order.
template <typename TX>
__global__ __launch_bounds__(256) void router_fwd_small_e(const TX* __restrict__ x, const TX* __restrict__ wr,
                                                         float* __restrict__ logits, int d, int E) {
  __shared__ float red[8][4];
  const int t = blockIdx.x, lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
  for (int e0 = 0; e0 < E; e0 += 8) {
    const int ne = E - e0 < 8 ? E - e0 : 8;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    if (sizeof(TX) == 2 && (E & 7) == 0 && (d & 7) == 0) {
      // bf16, whole groups of eight: 16-byte loads of eight columns of x and of each column's eight weights
      const uint16_t* xb = reinterpret_cast<const uint16_t*>(x);
      const uint16_t* wb = reinterpret_cast<const uint16_t*>(wr);
      for (int c8 = threadIdx.x * 8; c8 < d; c8 += 2048) {
        const uint4 xq = *reinterpret_cast<const uint4*>(xb + (size_t)t * d + c8);
        const uint32_t* xu = reinterpret_cast<const uint32_t*>(&xq);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float xv = (j & 1) ? bf16hi(xu[j >> 1]) : bf16lo(xu[j >> 1]);
          const uint4 wq = *reinterpret_cast<const uint4*>(wb + (size_t)(c8 + j) * E + e0);
          const uint32_t* wu = reinterpret_cast<const uint32_t*>(&wq);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[2 * i] += xv * bf16lo(wu[i]);
            acc[2 * i + 1] += xv * bf16hi(wu[i]);
          }
        }
      }
    } else {
      for (int c = threadIdx.x; c < d; c += 256) {
        const float xv = ldf(x, (size_t)t * d + c);
        const TX* w = wr + (size_t)c * E + e0;
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (i < ne) acc[i] += xv * ldf(w, i);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = wave_sum_f(acc[i]);
      if (lane == 0) red[i][wave] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < ne)
      logits[(size_t)t * E + e0 + threadIdx.x] = (red[threadIdx.x][0] + red[threadIdx.x][1]) + (red[threadIdx.x][2] + red[threadIdx.x][3]);
    __syncthreads();
  }
}

__global__ void round_to_bf16(const float* __restrict__ in, bf16_t* __restrict__ out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    out[i] = f32_to_bf16(in[i]);
}

// ---- fused backward of combine ------------------------------------------------------------
// One block per token.  dy[t] is read once; for each local slot the matching row of o is read,
// its dot product with dy[t] is reduced (lanes -> wavefront -> block, fixed order) and the
// gate-scaled row of d_o is written.  Bytes: (U + 2R) * d * b.
template <bool BF16>
__device__ __forceinline__ float dot_vec(u32x4 a, u32x4 b) {
  if (BF16) {
    float s = bf16lo(a.x) * bf16lo(b.x);
    s += bf16hi(a.x) * bf16hi(b.x);
    s += bf16lo(a.y) * bf16lo(b.y); s += bf16hi(a.y) * bf16hi(b.y);
    s += bf16lo(a.z) * bf16lo(b.z); s += bf16hi(a.z) * bf16hi(b.z);
    s += bf16lo(a.w) * bf16lo(b.w); s += bf16hi(a.w) * bf16hi(b.w);
    return s;
  } else {
    float s = __uint_as_float(a.x) * __uint_as_float(b.x);
    s += __uint_as_float(a.y) * __uint_as_float(b.y);
    s += __uint_as_float(a.z) * __uint_as_float(b.z);
    s += __uint_as_float(a.w) * __uint_as_float(b.w);
    return s;
  }
}
template <bool BF16>
__device__ __forceinline__ u32x4 scale_vec2(u32x4 v, float sc) {
  u32x4 r;
  if (BF16) {
    r.x = pack_bf16x2(bf16lo(v.x) * sc, bf16hi(v.x) * sc);
    r.y = pack_bf16x2(bf16lo(v.y) * sc, bf16hi(v.y) * sc);
    r.z = pack_bf16x2(bf16lo(v.z) * sc, bf16hi(v.z) * sc);
    r.w = pack_bf16x2(bf16lo(v.w) * sc, bf16hi(v.w) * sc);
  } else {
    r.x = __float_as_uint(__uint_as_float(v.x) * sc);
    r.y = __float_as_uint(__uint_as_float(v.y) * sc);
    r.z = __float_as_uint(__uint_as_float(v.z) * sc);
    r.w = __float_as_uint(__uint_as_float(v.w) * sc);
  }
  return r;
}

constexpr int CB_MAX_WAVES = 16;

template <bool BF16>
__global__ __launch_bounds__(1024) void combine_bwd_rows(const u32x4* __restrict__ dy, const u32x4* __restrict__ o,
                                                        int row_vecs, int k, const int32_t* __restrict__ inv,
                                                        const float* __restrict__ topk_w, u32x4* __restrict__ d_o,
                                                        float* __restrict__ dgate) {
  __shared__ float red[MOE_MAX_TOPK * CB_MAX_WAVES];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
  const int n_waves = blockDim.x / WAVE;
  const int32_t* irow = inv + (size_t)t * k;         // uniform address: scalar loads
  for (int i = tid; i < k * CB_MAX_WAVES; i += blockDim.x) red[i] = 0.f;
  __syncthreads();
  for (int c0 = 0; c0 < row_vecs; c0 += blockDim.x) {
    const int c = c0 + tid;
    const bool in = c < row_vecs;
    u32x4 v = {0u, 0u, 0u, 0u};
    bool loaded = false;
    for (int j = 0; j < k; ++j) {                     // ascending slot j; the branch is block-uniform
      const int row = irow[j];
      if (row < 0) continue;
      if (!loaded) {
        if (in) v = __builtin_nontemporal_load(dy + (size_t)t * row_vecs + c);
        loaded = true;
      }
      float part = 0.f;
      if (in) {
        const u32x4 ov = __builtin_nontemporal_load(o + (size_t)row * row_vecs + c);
        part = dot_vec<BF16>(v, ov);
        __builtin_nontemporal_store(scale_vec2<BF16>(v, topk_w[(size_t)t * k + j]), d_o + (size_t)row * row_vecs + c);
      }
      part = wave_sum_f(part);
      if (lane == 0) red[j * CB_MAX_WAVES + wave] += part;   // each wavefront owns its column
    }
  }
  __syncthreads();
  if (tid < k) {
    float s = 0.f;
    for (int w = 0; w < n_waves; ++w) s += red[tid * CB_MAX_WAVES + w];
    dgate[(size_t)t * k + tid] = s;
  }
}

// ---- gradient through the gate weights ----------------------------------------------------
// One wavefront per token; lane j < k holds slot j (its expert, logit and dgate); each lane owns
// the logit positions lane + 64*i and writes them with one coalesced store.
template <int VPL>
__global__ __launch_bounds__(256) void gate_bwd_kernel(const float* __restrict__ logits,
                                                      const int32_t* __restrict__ topk_idx,
                                                      const float* __restrict__ dgate, int T, int E, int k, int mode,
                                                      float* __restrict__ dlogits) {
  const int lane = lane_id();
  const int wave = threadIdx.x / WAVE;
  const int waves_per_block = blockDim.x / WAVE;
  for (int t = blockIdx.x * waves_per_block + wave; t < T; t += gridDim.x * waves_per_block) {
    const float* row = logits + (size_t)t * E;
    const bool act = lane < k;
    int my_idx = act ? topk_idx[(size_t)t * k + lane] : -1;
    if (act) my_idx = my_idx < 0 ? 0 : (my_idx >= E ? E - 1 : my_idx);   // a corrupt index must not read out of bounds
    const float my_dg = act ? dgate[(size_t)t * k + lane] : 0.f;
    const float my_logit = act ? row[my_idx] : 0.f;
    float out[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) out[i] = 0.f;
    float d_sel = 0.f;
    if (mode == MOE_GATE_SOFTMAX_RENORM) {
      const float top = __shfl(my_logit, 0, WAVE);          // slot 0 holds the largest logit
      const float ex = act ? expf(my_logit - top) : 0.f;
      const float w = ex / wave_sum_f(ex);
      const float c = wave_sum_f(w * my_dg);
      d_sel = w * (my_dg - c);
    } else if (mode == MOE_GATE_SIGMOID_RENORM) {
      const float sg = act ? 1.0f / (1.0f + expf(-my_logit)) : 0.f;
      const float S = wave_sum_f(sg);
      const float c = wave_sum_f(sg / S * my_dg);
      d_sel = (my_dg - c) / S * sg * (1.0f - sg);
    } else {
      float v[VPL];
      float m = -INFINITY;
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
        const int e = lane + i * WAVE;
        v[i] = e < E ? row[e] : -INFINITY;
        m = fmaxf(m, v[i]);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, WAVE));
      float den = 0.f;
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
        v[i] = lane + i * WAVE < E ? expf(v[i] - m) : 0.f;
        den += v[i];
      }
      den = wave_sum_f(den);
      const float p_sel = act ? expf(my_logit - m) / den : 0.f;
      const float inner = wave_sum_f(p_sel * my_dg);
      d_sel = p_sel * (my_dg - inner);
#pragma unroll
      for (int i = 0; i < VPL; ++i) out[i] = -(v[i] / den) * inner;
    }
    for (int j = 0; j < k; ++j) {
      const int e = __shfl(my_idx, j, WAVE);
      const float dv = __shfl(d_sel, j, WAVE);
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (lane + i * WAVE == e) out[i] = dv;
    }
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const int e = lane + i * WAVE;
      if (e < E) dlogits[(size_t)t * E + e] = out[i];
    }
  }
}

inline int tiles(int n, int t) { return (n + t - 1) / t; }

// split of the token contraction for the plain path: enough blocks to fill the chip, chunk sums
// bounded to 64 MB
int valu_splits(int T, int d, int E) {
  const long long blocks = (long long)tiles(d, TM) * tiles(E, TN);
  long long s = (4LL * device_cu_count() + blocks - 1) / blocks;
  const long long by_bytes = (64LL << 20) / ((long long)d * E * 4);
  if (s > by_bytes) s = by_bytes;
  if (s > tiles(T, 4 * TK)) s = tiles(T, 4 * TK);
  if (s > 64) s = 64;
  return s < 1 ? 1 : (int)s;
}

inline bool mfma_shape(int dtype, int T, int d, int E) {
  return dtype == MOE_BF16 && T > 0 && E % 64 == 0 && d % 64 == 0;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

size_t router_ws_bytes(int dtype, int T, int d, int E) {
  size_t b = 256;                                           // ticket counters
  if (mfma_shape(dtype, T, d, E)) {
    // backward: dlogits rounded to bf16 + the chunk sums of dWr; forward: the logits of each range
    // of a cut contraction (the two calls use the same bytes one after the other)
    const size_t bwd = align256((size_t)T * E * 2) + align256((size_t)router_dw_splits(T, d, E) * d * E * 4);
    const int fs = router_fwd_splits(T, d, E);
    const size_t fwd = fs > 1 ? align256((size_t)fs * T * E * 4) : 0;
    b += bwd > fwd ? bwd : fwd;
  } else {
    b += align256((size_t)valu_splits(T, d, E) * d * E * 4);
  }
  return b;
}

int launch_router_fwd(const void* x, const void* wr, int dtype, int T, int d, int E, float* logits, void* ws,
                      hipStream_t s) {
  if (T == 0) return MOE_OK;
  if (mfma_shape(dtype, T, d, E)) {
    const int splits = router_fwd_splits(T, d, E);
    float* partial = (float*)((char*)ws + 256);
    int rc = launch_router_fwd_bf16(x, wr, T, d, E, logits, partial, splits, (int32_t*)ws, s);
    if (rc || splits == 1) return rc;
    ProfScope prof(MOE_K_ROUTER_FWD, s);
    hipLaunchKernelGGL((reduce_chunks<float>), dim3(device_cu_count() * 4), dim3(256), 0, s, partial, splits, (size_t)T * E,
                       logits, 0);
    HIP_CHECK_LAUNCH();
    return MOE_OK;
  }
  ProfScope prof(MOE_K_ROUTER_FWD, s);
  if (E <= 64) {
    if (dtype == MOE_BF16)
      hipLaunchKernelGGL((router_fwd_small_e<bf16_t>), dim3(T), dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)wr, logits, d, E);
    else
      hipLaunchKernelGGL((router_fwd_small_e<float>), dim3(T), dim3(256), 0, s, (const float*)x, (const float*)wr, logits, d, E);
  } else {
    dim3 grid(tiles(E, TN), tiles(T, TM)), blk(256);
    if (dtype == MOE_BF16)
      hipLaunchKernelGGL((gemm_rows_valu<bf16_t, bf16_t, float>), grid, blk, 0, s, (const bf16_t*)x, d, (const bf16_t*)wr,
                         (long)E, 1L, logits, E, T, E, d, 0);
    else
      hipLaunchKernelGGL((gemm_rows_valu<float, float, float>), grid, blk, 0, s, (const float*)x, d, (const float*)wr,
                         (long)E, 1L, logits, E, T, E, d, 0);
  }
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_combine_bwd(const void* dy, const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                       const float* topk_w, void* d_o, float* dgate, hipStream_t s) {
  if (T == 0) return MOE_OK;
  ProfScope prof(MOE_K_COMBINE_BWD, s);
  const int row_vecs = dtype == MOE_BF16 ? d / 8 : d / 4;
  int bs = (row_vecs + WAVE - 1) / WAVE * WAVE;
  if (bs > 1024) bs = 1024;
  if (bs < 64) bs = 64;
  if (dtype == MOE_BF16)
    hipLaunchKernelGGL((combine_bwd_rows<true>), dim3(T), dim3(bs), 0, s, (const u32x4*)dy, (const u32x4*)o, row_vecs, k,
                       inv, topk_w, (u32x4*)d_o, dgate);
  else
    hipLaunchKernelGGL((combine_bwd_rows<false>), dim3(T), dim3(bs), 0, s, (const u32x4*)dy, (const u32x4*)o, row_vecs, k,
                       inv, topk_w, (u32x4*)d_o, dgate);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_gate_bwd(const float* logits, const int32_t* topk_idx, const float* dgate, int T, int E, int k,
                    int gate_mode, float* dlogits, hipStream_t s) {
  if (T == 0) return MOE_OK;
  ProfScope prof(MOE_K_GATE_BWD, s);
  const int wpb = 4;
  int blocks = (T + wpb - 1) / wpb;
  const int maxb = device_cu_count() * 8;
  if (blocks > maxb) blocks = maxb;
  const int vpl = (E + WAVE - 1) / WAVE;
#define GATE_CASE(V)                                                                                          \
  hipLaunchKernelGGL(gate_bwd_kernel<V>, dim3(blocks), dim3(256), 0, s, logits, topk_idx, dgate, T, E, k, gate_mode, \
                     dlogits)
  if (vpl <= 1) GATE_CASE(1);
  else if (vpl <= 2) GATE_CASE(2);
  else if (vpl <= 4) GATE_CASE(4);
  else if (vpl <= 8) GATE_CASE(8);
  else GATE_CASE(16);
#undef GATE_CASE
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_router_bwd(const void* x, const void* wr, const float* dlogits, int dtype, int T, int d, int E, void* dwr,
                      int dwr_acc, void* dx, int dx_acc, void* ws, hipStream_t s) {
  int32_t* sched = (int32_t*)ws;
  char* base = (char*)ws + 256;
  const size_t n_w = (size_t)d * E;
  const int red_blocks = device_cu_count() * 4;
  int rc;
  if (mfma_shape(dtype, T, d, E)) {
    bf16_t* dlb = (bf16_t*)base;
    float* partial = (float*)(base + align256((size_t)T * E * 2));
    if ((rc = launch_zero_words(sched, 16, s))) return rc;
    {
      ProfScope prof(dwr ? MOE_K_ROUTER_DW : MOE_K_ROUTER_DX, s);
      hipLaunchKernelGGL(round_to_bf16, dim3(red_blocks), dim3(256), 0, s, dlogits, dlb, (size_t)T * E);
      HIP_CHECK_LAUNCH();
    }
    if (dwr) {
      const int splits = router_dw_splits(T, d, E);
      if ((rc = launch_router_dw_bf16(x, dlb, T, d, E, partial, splits, sched, s))) return rc;
      ProfScope prof(MOE_K_ROUTER_DW, s);
      hipLaunchKernelGGL((reduce_chunks<bf16_t>), dim3(red_blocks), dim3(256), 0, s, partial, splits, n_w, (bf16_t*)dwr,
                         dwr_acc);
      HIP_CHECK_LAUNCH();
    }
    if (dx) return launch_router_dx_bf16(dlb, wr, T, d, E, dx, dx_acc, sched + 8, s);
    return MOE_OK;
  }
  float* partial = (float*)base;
  if (dwr) {
    const int splits = T > 0 ? valu_splits(T, d, E) : 0;
    if (splits > 0) {
      ProfScope prof(MOE_K_ROUTER_DW, s);
      const int chunk = (T + splits - 1) / splits;
      dim3 grid(tiles(E, TN), tiles(d, TM), splits), blk(256);
      if (dtype == MOE_BF16)
        hipLaunchKernelGGL((gemm_tn_valu<bf16_t>), grid, blk, 0, s, (const bf16_t*)x, d, dlogits, E, partial, d, E, T, chunk);
      else
        hipLaunchKernelGGL((gemm_tn_valu<float>), grid, blk, 0, s, (const float*)x, d, dlogits, E, partial, d, E, T, chunk);
      HIP_CHECK_LAUNCH();
    }
    if (dtype == MOE_BF16)
      hipLaunchKernelGGL((reduce_chunks<bf16_t>), dim3(red_blocks), dim3(256), 0, s, partial, splits, n_w, (bf16_t*)dwr, dwr_acc);
    else
      hipLaunchKernelGGL((reduce_chunks<float>), dim3(red_blocks), dim3(256), 0, s, partial, splits, n_w, (float*)dwr, dwr_acc);
    HIP_CHECK_LAUNCH();
  }
  if (dx && T > 0) {
    ProfScope prof(MOE_K_ROUTER_DX, s);
    if (E <= 64) {
      // a handful of experts: per-token dot products against contiguous weight rows
      const int col_groups = tiles(d, 1024);
      if ((long long)col_groups * T >= (1ll << 31)) return MOE_EUNSUPPORTED;
      dim3 grid((unsigned)(col_groups * T)), blk(256);
      if (dtype == MOE_BF16)
        hipLaunchKernelGGL((router_dx_small_e<bf16_t>), grid, blk, 0, s, dlogits, (const bf16_t*)wr, (bf16_t*)dx, d, E, dx_acc, col_groups);
      else
        hipLaunchKernelGGL((router_dx_small_e<float>), grid, blk, 0, s, dlogits, (const float*)wr, (float*)dx, d, E, dx_acc, col_groups);
    } else {
      // dx[t,n] (+)= sum_e dl[t,e] * Wr[n,e] : B(k = e, n) = Wr[n*E + e]
      dim3 grid(tiles(d, TN), tiles(T, TM)), blk(256);
      if (dtype == MOE_BF16)
        hipLaunchKernelGGL((gemm_rows_valu<float, bf16_t, bf16_t>), grid, blk, 0, s, dlogits, E, (const bf16_t*)wr, 1L, (long)E,
                           (bf16_t*)dx, d, T, d, E, dx_acc);
      else
        hipLaunchKernelGGL((gemm_rows_valu<float, float, float>), grid, blk, 0, s, dlogits, E, (const float*)wr, 1L, (long)E,
                           (float*)dx, d, T, d, E, dx_acc);
    }
    HIP_CHECK_LAUNCH();
  }
  return MOE_OK;
}
