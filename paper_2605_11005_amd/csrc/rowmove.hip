// Row movers: dispatch (token order -> expert order) and combine (expert order -> token
// order, gate-weighted).  Both are token-major (a token's row is split over a few blocks), so every row
// of x / o is read exactly once and every row of xp / y is written exactly once:
//   dispatch : read x[t] once (skipped when the token has no local slot), write it to each
//              of the token's local rows            -> (U + R) * d * b bytes
//   combine  : read the token's local rows, write y[t] once (zeros when none)
//                                                   -> (R + T) * d * b bytes
// Accesses are 16 bytes per lane and one vector per thread: on this chip a plain copy is fastest
// with the largest possible number of small threads.  Dispatch numbers its blocks row-segment
// fastest, token next, so that blocks resident together work on consecutive 2 KB pieces of the
// same rows (source and destinations): DRAM pages are used while they are open.
#include "common.h"
#include "kernels.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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

// row_vecs = number of 16-byte vectors per row; one vector per thread.
// dispatch: 1-D grid of T * n_seg blocks of 128 threads, block = (token t, segment of 128 vectors),
//   segment fastest.  Measured at T = 32768, d = 7168 (896 vectors = 7 segments): 6.3 TB/s against
//   5.4 TB/s with the token index fastest and 256-thread blocks (whose fourth block is half empty).
// combine: the same numbering and block size (6.5 TB/s against 6.1-6.3 TB/s with one block per token row).
constexpr int DISPATCH_BLOCK = 128;
constexpr int COMBINE_BLOCK = 128;

template <bool BF16, bool SCALED>
__global__ __launch_bounds__(DISPATCH_BLOCK) void dispatch_rows(const u32x4* __restrict__ x, int T, int row_vecs, int n_seg,
                                                    int k, const int32_t* __restrict__ inv,
                                                    const float* __restrict__ row_scale,
                                                    u32x4* __restrict__ xp) {
  const int t = blockIdx.x / n_seg;
  const int c = (blockIdx.x - t * n_seg) * DISPATCH_BLOCK + threadIdx.x;
  const int32_t* irow = inv + (size_t)t * k;         // uniform address: scalar loads
  int first = -1;
  for (int j = 0; j < k; ++j)
    if (irow[j] >= 0) { first = j; break; }
  if (first < 0 || c >= row_vecs) return;             // token without a local slot: nothing is read
  const u32x4 v = __builtin_nontemporal_load(x + (size_t)t * row_vecs + c);
  for (int j = first; j < k; ++j) {
    const int row = irow[j];
    if (row < 0) continue;
    const float sc = SCALED ? row_scale[(size_t)t * k + j] : 1.0f;
    const u32x4 o = SCALED ? scale_vec<BF16>(v, sc) : v;
    __builtin_nontemporal_store(o, xp + (size_t)row * row_vecs + c);
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
__global__ __launch_bounds__(COMBINE_BLOCK) void combine_rows(const u32x4* __restrict__ o, int T, int row_vecs, int n_seg,
                                                   int k, const int32_t* __restrict__ inv,
                                                   const float* __restrict__ topk_w,
                                                   u32x4* __restrict__ y) {
  const int t = blockIdx.x / n_seg;
  const int c = (blockIdx.x - t * n_seg) * COMBINE_BLOCK + threadIdx.x;
  if (c >= row_vecs) return;
  const int32_t* irow = inv + (size_t)t * k;         // uniform address: scalar loads
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int j = 0; j < k; ++j) {                       // ascending slot j
    const int row = irow[j];
    if (row < 0) continue;
    const float w = topk_w ? topk_w[(size_t)t * k + j] : 1.0f;
    const u32x4 v = __builtin_nontemporal_load(o + (size_t)row * row_vecs + c);
    fma_vec<BF16>(acc, v, w);
  }
  __builtin_nontemporal_store(pack_acc<BF16>(acc), y + (size_t)t * row_vecs + c);
}

}  // namespace

int launch_dispatch_rows(const void* x, int dtype, int T, int d, int k, const int32_t* inv,
                         const float* row_scale, void* xp, hipStream_t s) {
  if (T == 0) return MOE_OK;
  ProfScope prof(MOE_K_DISPATCH, s);
  const int row_vecs = dtype == MOE_BF16 ? d / 8 : d / 4;
  const int n_seg = (row_vecs + DISPATCH_BLOCK - 1) / DISPATCH_BLOCK;
  if ((long long)T * n_seg >= (1ll << 31)) return MOE_EUNSUPPORTED;      // 1-D grid limit (checked by the entry point too)
  dim3 grid((unsigned)(T * n_seg)), block(DISPATCH_BLOCK);
  const u32x4* xs = (const u32x4*)x;
  u32x4* xd = (u32x4*)xp;
  if (dtype == MOE_BF16) {
    if (row_scale) hipLaunchKernelGGL((dispatch_rows<true, true>), grid, block, 0, s, xs, T, row_vecs, n_seg, k, inv, row_scale, xd);
    else hipLaunchKernelGGL((dispatch_rows<true, false>), grid, block, 0, s, xs, T, row_vecs, n_seg, k, inv, row_scale, xd);
  } else {
    if (row_scale) hipLaunchKernelGGL((dispatch_rows<false, true>), grid, block, 0, s, xs, T, row_vecs, n_seg, k, inv, row_scale, xd);
    else hipLaunchKernelGGL((dispatch_rows<false, false>), grid, block, 0, s, xs, T, row_vecs, n_seg, k, inv, row_scale, xd);
  }
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

int launch_combine_rows(const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                        const float* topk_w, void* y, hipStream_t s) {
  if (T == 0) return MOE_OK;
  ProfScope prof(MOE_K_COMBINE, s);
  const int row_vecs = dtype == MOE_BF16 ? d / 8 : d / 4;
  const int n_seg = (row_vecs + COMBINE_BLOCK - 1) / COMBINE_BLOCK;
  if ((long long)T * n_seg >= (1ll << 31)) return MOE_EUNSUPPORTED;      // 1-D grid limit (checked by the entry point too)
  dim3 grid((unsigned)(T * n_seg)), block(COMBINE_BLOCK);
  if (dtype == MOE_BF16)
    hipLaunchKernelGGL((combine_rows<true>), grid, block, 0, s, (const u32x4*)o, T, row_vecs, n_seg, k, inv, topk_w, (u32x4*)y);
  else
    hipLaunchKernelGGL((combine_rows<false>), grid, block, 0, s, (const u32x4*)o, T, row_vecs, n_seg, k, inv, topk_w, (u32x4*)y);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}
