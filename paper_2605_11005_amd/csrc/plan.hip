// The dispatch plan: a stable counting sort of the flat slots s = t*k + j by local expert.
//
// Three small kernels, no order-dependent atomics, so perm/inv are unique and reproducible:
//   1. plan_hist    -- every wavefront owns CHUNK consecutive slots and writes the histogram
//                      of their local experts to ws_hist[e][chunk] (chunks contiguous per expert,
//                      so that the scan reads coalesced).
//   2. plan_scan    -- one block, one wavefront per expert: an exclusive running sum over the chunks
//                      (-> first row of that expert inside each chunk), then the exclusive
//                      prefix over experts (-> offsets), clamped to cap with a status word.
//   3. plan_scatter -- every wavefront revisits its chunk in slot order; within each group
//                      of 64 slots the rank among equal keys comes from a ballot + popcount
//                      of the lower lanes, and a per-wave LDS counter carries it forward.
#include "common.h"
#include "kernels.h"

#include <mutex>

namespace {

constexpr int CHUNK = 512;   // slots per wavefront

__global__ __launch_bounds__(64) void plan_hist(const int32_t* __restrict__ topk_idx, int n_slots, int e_lo,
                                               int e_cnt, int32_t* __restrict__ ws_hist) {
  extern __shared__ int32_t h[];
  const int lane = threadIdx.x;
  for (int i = lane; i < e_cnt; i += WAVE) h[i] = 0;
  __syncthreads();
  const int base = blockIdx.x * CHUNK;
  for (int i = lane; i < CHUNK; i += WAVE) {
    int s = base + i;
    if (s < n_slots) {
      int le = topk_idx[s] - e_lo;
      if (le >= 0 && le < e_cnt) atomicAdd(&h[le], 1);
    }
  }
  __syncthreads();
  for (int i = lane; i < e_cnt; i += WAVE) ws_hist[(size_t)i * gridDim.x + blockIdx.x] = h[i];   // [expert][chunk]
}

// ws_hist[e][c] becomes the first row (before the expert's offset is added) of expert e in chunk c.
// One wavefront per expert: 64 chunks at a time, exclusive scan by lane shuffles, carry across
// groups of 64.
__global__ __launch_bounds__(1024) void plan_scan(int32_t* __restrict__ ws_hist, int n_chunks, int e_cnt, int cap,
                                                 int32_t* __restrict__ offsets, int32_t* __restrict__ status) {
  __shared__ int32_t total[MOE_MAX_LOCAL + 1];
  const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE, n_waves = blockDim.x / WAVE;
  for (int e = wave; e < e_cnt; e += n_waves) {
    int carry = 0;
    // eight groups of 64 chunks per batch: all loads of a batch are issued before the first scan,
    // so a batch costs one memory round trip instead of eight
    for (int b0 = 0; b0 < n_chunks; b0 += 8 * WAVE) {
      int v[8];
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        const int c = b0 + g * WAVE + lane;
        v[g] = c < n_chunks ? ws_hist[(size_t)e * n_chunks + c] : 0;
      }
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        const int c = b0 + g * WAVE + lane;
        int incl = v[g];
#pragma unroll
        for (int off = 1; off < WAVE; off <<= 1) {
          int t = __shfl_up(incl, off, WAVE);
          if (lane >= off) incl += t;
        }
        if (c < n_chunks) ws_hist[(size_t)e * n_chunks + c] = carry + incl - v[g];
        carry += __shfl(incl, WAVE - 1, WAVE);
      }
    }
    if (lane == 0) total[e] = carry;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < e_cnt; ++i) {
      int v = total[i];
      total[i] = run;
      run += v;
    }
    total[e_cnt] = run;
    *status = run > cap ? 1 : 0;
  }
  __syncthreads();
  // unclamped expert bases stay in ws (after the chunk table) for the scatter pass
  int32_t* ebase = ws_hist + (size_t)n_chunks * e_cnt;
  for (int i = threadIdx.x; i <= e_cnt; i += blockDim.x) {
    int v = total[i];
    ebase[i] = v;
    offsets[i] = v < cap ? v : cap;
  }
}

__global__ __launch_bounds__(64) void plan_scatter(const int32_t* __restrict__ topk_idx, int n_slots, int e_lo,
                                                  int e_cnt, int cap, const int32_t* __restrict__ ws_hist,
                                                  int n_chunks, int32_t* __restrict__ perm,
                                                  int32_t* __restrict__ inv) {
  extern __shared__ int32_t run[];
  const int lane = threadIdx.x;
  const int32_t* ebase = ws_hist + (size_t)n_chunks * e_cnt;
  for (int i = lane; i < e_cnt; i += WAVE) run[i] = ebase[i] + ws_hist[(size_t)i * n_chunks + blockIdx.x];
  __syncthreads();
  const int base = blockIdx.x * CHUNK;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  for (int step = 0; step < CHUNK; step += WAVE) {
    const int s = base + step + lane;
    int le = -1;
    if (s < n_slots) {
      le = topk_idx[s] - e_lo;
      if (le < 0 || le >= e_cnt) le = -1;
    }
    int row = -1;
    unsigned long long todo = __ballot(le >= 0);
    while (todo) {                                   // wave-uniform loop over distinct keys
      const int leader = __ffsll((long long)todo) - 1;
      const int key = __shfl(le, leader, WAVE);
      const unsigned long long same = __ballot(le == key);
      const int first = run[key];
      if (le == key) row = first + __popcll(same & lt_mask);
      __syncthreads();                               // everyone has read run[key]
      if (lane == leader) run[key] = first + __popcll(same);
      __syncthreads();
      todo &= ~same;
    }
    if (s < n_slots) {
      if (row >= cap) row = -1;                      // dropped: caller's cap was too small
      inv[s] = row;
      if (row >= 0) perm[row] = s;
    }
  }
}

}  // namespace

// ---- plan scratch that lives in the code object, for callers that cannot allocate ---------
// One array per GPU (each device that loads the library holds its own copy at its own address
// until the process ends).  Host code never passes the array's name to a kernel: the name is a
// host-side stand-in, the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_PLAN_BYTES];

namespace {
std::mutex g_scratch_lock;
void* g_scratch_ptr[64] = {};
}  // namespace

int plan_static_scratch(void** ptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MOE_EHIP;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MOE_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return MOE_OK;
}

size_t plan_ws_bytes(int T, int k, int e_cnt) {
  size_t n_slots = (size_t)T * (size_t)k;
  size_t n_chunks = (n_slots + CHUNK - 1) / CHUNK;
  // status word (own 256-byte line) + chunk table + expert bases
  return 256 + (n_chunks * (size_t)e_cnt + (size_t)e_cnt + 1) * sizeof(int32_t);
}

int launch_plan(const int32_t* topk_idx, int T, int k, int e_lo, int e_cnt, int32_t* offsets,
                int32_t* perm, int32_t* inv, int cap, void* ws, int32_t* status_out, hipStream_t s) {
  ProfScope prof(MOE_K_PLAN, s);
  int32_t* status = status_out ? status_out : (int32_t*)ws;
  int32_t* ws_hist = (int32_t*)((char*)ws + 256);
  const long long n_slots = (long long)T * k;
  const int n_chunks = (int)((n_slots + CHUNK - 1) / CHUNK);
  size_t shm = (size_t)(e_cnt > 0 ? e_cnt : 1) * sizeof(int32_t);
  if (n_chunks > 0) {
    hipLaunchKernelGGL(plan_hist, dim3(n_chunks), dim3(64), shm, s, topk_idx, (int)n_slots, e_lo, e_cnt, ws_hist);
    HIP_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL(plan_scan, dim3(1), dim3(1024), 0, s, ws_hist, n_chunks, e_cnt, cap, offsets, status);
  HIP_CHECK_LAUNCH();
  if (n_chunks > 0) {
    hipLaunchKernelGGL(plan_scatter, dim3(n_chunks), dim3(64), shm, s, topk_idx, (int)n_slots, e_lo, e_cnt, cap,
                       ws_hist, n_chunks, perm, inv);
    HIP_CHECK_LAUNCH();
  }
  return MOE_OK;
}
