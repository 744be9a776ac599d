// fp32 expert FFNs (correctness-grade path for the small all-fp32 configuration).
// Plain LDS-tiled FMA GEMMs, 64x64 output tile per 256-thread block, 4x4 per thread,
// fp32 accumulation in ascending-k order.  The bf16 MFMA path is in expert_bf16.hip.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

// Ragged-M grouped GEMM: for expert e and its rows r in [off[e], off[e+1]):
//   C[r, n] = beta*C[r,n] + sum_k A[r,k] * B_e(k,n),   B_e(k,n) = B[e*b_es + k*b_rs + n*b_cs]
// grid.x = N tiles, grid.y = upper bound on M tiles (ceil(cap/TM) + e_cnt).
__global__ __launch_bounds__(256) void gemm_rows_f32(const float* __restrict__ A, int lda, const float* __restrict__ B,
                                                    long b_es, long b_rs, long b_cs, float* __restrict__ C,
                                                    int ldc, int N, int K, int e_cnt,
                                                    const int32_t* __restrict__ off, int beta) {
  // locate this block's (expert, m-tile)
  int mt = blockIdx.y, e = 0, lo = 0, hi = 0;
  for (; e < e_cnt; ++e) {
    lo = off[e]; hi = off[e + 1];
    int tiles = (hi - lo + TM - 1) / TM;
    if (mt < tiles) break;
    mt -= tiles;
  }
  if (e >= e_cnt) return;
  const int row0 = lo + mt * TM, col0 = blockIdx.x * TN;
  __shared__ float sa[TK][TM + 1], sb[TK][TN + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  const float* Be = B + (size_t)e * b_es;
  for (int k0 = 0; k0 < K; k0 += TK) {
    for (int i = threadIdx.x; i < TM * TK; i += 256) {
      int m = i / TK, kk = i % TK;
      int r = row0 + m, kidx = k0 + kk;
      sa[kk][m] = (r < hi && kidx < K) ? A[(size_t)r * lda + kidx] : 0.f;
    }
    for (int i = threadIdx.x; i < TN * TK; i += 256) {
      int n, kk;
      if (b_cs == 1) { n = i % TN; kk = i / TN; } else { kk = i % TK; n = i / TK; }
      int c = col0 + n, kidx = k0 + kk;
      sb[kk][n] = (c < N && kidx < K) ? Be[(size_t)kidx * b_rs + (size_t)c * b_cs] : 0.f;
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
    int r = row0 + ty * 4 + i;
    if (r >= hi) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = col0 + tx * 4 + j;
      if (c < N) {
        size_t idx = (size_t)r * ldc + c;
        C[idx] = beta ? C[idx] + acc[i][j] : acc[i][j];
      }
    }
  }
}

// Ragged-K grouped GEMM (weight gradients): C_e[i,j] = beta*C_e[i,j] + sum_{r in expert e} P[r,i]*Q[r,j]
// grid = (N tiles, M tiles, e_cnt)
__global__ __launch_bounds__(256) void gemm_wgrad_f32(const float* __restrict__ P, int ldp, const float* __restrict__ Q,
                                                     int ldq, float* __restrict__ C, int M, int N,
                                                     const int32_t* __restrict__ off, int beta) {
  const int e = blockIdx.z;
  const int lo = off[e], hi = off[e + 1];
  const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TN;
  __shared__ float sa[TK][TM + 1], sb[TK][TN + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int r0 = lo; r0 < hi; r0 += TK) {
    for (int t = threadIdx.x; t < TM * TK; t += 256) {
      int m = t % TM, kk = t / TM;
      int r = r0 + kk, i = i0 + m;
      sa[kk][m] = (r < hi && i < M) ? P[(size_t)r * ldp + i] : 0.f;
    }
    for (int t = threadIdx.x; t < TN * TK; t += 256) {
      int n = t % TN, kk = t / TN;
      int r = r0 + kk, j = j0 + n;
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
  float* Ce = C + (size_t)e * M * N;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int ii = i0 + ty * 4 + i;
    if (ii >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int jj = j0 + tx * 4 + j;
      if (jj < N) {
        size_t idx = (size_t)ii * N + jj;
        Ce[idx] = beta ? Ce[idx] + acc[i][j] : acc[i][j];
      }
    }
  }
}

// a = silu(h1) * h3 on rows [0, R), R = off[e_cnt]
__global__ void swiglu_fwd_f32(const float* __restrict__ h1, const float* __restrict__ h3, float* __restrict__ a,
                               int f, const int32_t* __restrict__ off, int e_cnt) {
  const size_t n = (size_t)off[e_cnt] * f;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float z = h1[i];
    a[i] = (z / (1.0f + expf(-z))) * h3[i];
  }
}

// in: dA (in dh1 buffer), h1, h3.  out: a, dH1 (in place of dA), dH3
__global__ void swiglu_bwd_f32(const float* __restrict__ h1, const float* __restrict__ h3, float* __restrict__ a,
                               float* __restrict__ dh1, float* __restrict__ dh3, int f,
                               const int32_t* __restrict__ off, int e_cnt) {
  const size_t n = (size_t)off[e_cnt] * f;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float z = h1[i], g = h3[i], da = dh1[i];
    float sg = 1.0f / (1.0f + expf(-z));
    float sl = z * sg;
    a[i] = sl * g;
    dh1[i] = da * g * (sg * (1.0f + z * (1.0f - sg)));
    dh3[i] = da * sl;
  }
}

inline int m_tiles_bound(int cap, int e_cnt) { return (cap + TM - 1) / TM + e_cnt; }

}  // namespace

int launch_expert_fwd_f32(const float* xp, int cap, int d, int f, int e_cnt, const int32_t* offsets,
                          const float* w1, const float* w3, const float* w2, float* h1, float* h3,
                          float* o, float* a_ws, hipStream_t s) {
  if (cap == 0 || e_cnt == 0) return MOE_OK;
  const int mtb = m_tiles_bound(cap, e_cnt);
  dim3 blk(256);
  hipLaunchKernelGGL(gemm_rows_f32, dim3((f + TN - 1) / TN, mtb), blk, 0, s, xp, d, w1, (long)d * f, (long)f, 1L, h1, f, f, d, e_cnt, offsets, 0);
  HIP_CHECK_LAUNCH();
  hipLaunchKernelGGL(gemm_rows_f32, dim3((f + TN - 1) / TN, mtb), blk, 0, s, xp, d, w3, (long)d * f, (long)f, 1L, h3, f, f, d, e_cnt, offsets, 0);
  HIP_CHECK_LAUNCH();
  hipLaunchKernelGGL(swiglu_fwd_f32, dim3(device_cu_count() * 4), dim3(256), 0, s, h1, h3, a_ws, f, offsets, e_cnt);
  HIP_CHECK_LAUNCH();
  hipLaunchKernelGGL(gemm_rows_f32, dim3((d + TN - 1) / TN, mtb), blk, 0, s, a_ws, f, w2, (long)f * d, (long)d, 1L, o, d, d, f, e_cnt, offsets, 0);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_expert_bwd_f32(const float* xp, const float* h1, const float* h3, const float* a_in, const float* d_o, int cap,
                          int d, int f, int e_cnt, const int32_t* offsets, const float* w1,
                          const float* w3, const float* w2, float* dxp, float* dw1, float* dw3,
                          float* dw2, int accumulate, float* ws, hipStream_t s) {
  if (e_cnt == 0) return MOE_OK;
  float* a = ws;
  float* dh1 = ws + (size_t)cap * f;
  float* dh3 = ws + 2 * (size_t)cap * f;
  dim3 blk(256);
  if (cap > 0) {
    const int mtb = m_tiles_bound(cap, e_cnt);
    // dA = d_o W2^T : B_e(k = col of d, n = row of f) = W2[e][n][k]
    hipLaunchKernelGGL(gemm_rows_f32, dim3((f + TN - 1) / TN, mtb), blk, 0, s, d_o, d, w2, (long)f * d, 1L, (long)d, dh1, f, f, d, e_cnt, offsets, 0);
    HIP_CHECK_LAUNCH();
    hipLaunchKernelGGL(swiglu_bwd_f32, dim3(device_cu_count() * 4), dim3(256), 0, s, h1, h3, a, dh1, dh3, f, offsets, e_cnt);
    HIP_CHECK_LAUNCH();
    // dxp = dH1 W1^T + dH3 W3^T : B_e(k = col of f, n = row of d) = W1[e][n][k]
    hipLaunchKernelGGL(gemm_rows_f32, dim3((d + TN - 1) / TN, mtb), blk, 0, s, dh1, f, w1, (long)d * f, 1L, (long)f, dxp, d, d, f, e_cnt, offsets, 0);
    HIP_CHECK_LAUNCH();
    hipLaunchKernelGGL(gemm_rows_f32, dim3((d + TN - 1) / TN, mtb), blk, 0, s, dh3, f, w3, (long)d * f, 1L, (long)f, dxp, d, d, f, e_cnt, offsets, 1);
    HIP_CHECK_LAUNCH();
  }
  const int beta = accumulate ? 1 : 0;
  // dW2 takes the activation the forward kept, if the caller passed it, else the one recomputed above
  hipLaunchKernelGGL(gemm_wgrad_f32, dim3((d + TN - 1) / TN, (f + TM - 1) / TM, e_cnt), blk, 0, s, a_in ? a_in : a, f, d_o, d, dw2, f, d, offsets, beta);
  HIP_CHECK_LAUNCH();
  hipLaunchKernelGGL(gemm_wgrad_f32, dim3((f + TN - 1) / TN, (d + TM - 1) / TM, e_cnt), blk, 0, s, xp, d, dh1, f, dw1, d, f, offsets, beta);
  HIP_CHECK_LAUNCH();
  hipLaunchKernelGGL(gemm_wgrad_f32, dim3((f + TN - 1) / TN, (d + TM - 1) / TM, e_cnt), blk, 0, s, xp, d, dh3, f, dw3, d, f, offsets, beta);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}
