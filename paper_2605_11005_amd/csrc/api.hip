// The C ABI (include/moe.h): argument validation on the host, then kernel launches.
#include "kernels.h"

#include <algorithm>
#include <mutex>
#include <vector>

namespace {

inline bool bad_dtype(int dtype) { return dtype != MOE_F32 && dtype != MOE_BF16; }
inline size_t esize(int dtype) { return dtype == MOE_BF16 ? 2 : 4; }
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

int shape_check_expert(int dtype, int cap, int d, int f, int e_cnt) {
  if (bad_dtype(dtype) || cap < 0 || d <= 0 || f <= 0 || e_cnt < 0) return MOE_EINVAL;
  if (e_cnt > MOE_MAX_LOCAL) return MOE_EUNSUPPORTED;
  if (dtype == MOE_BF16 && (d % 64 || f % 64)) return MOE_EUNSUPPORTED;
  if (dtype == MOE_F32 && (d % 4 || f % 4)) return MOE_EUNSUPPORTED;
  // 32-bit row*ld products inside a tile and 31-bit element counts per activation tensor
  if ((long long)cap * (d > f ? d : f) >= (1ll << 40)) return MOE_EUNSUPPORTED;
  if ((long long)(d > f ? d : f) * 256 >= (1ll << 31)) return MOE_EUNSUPPORTED;
  // the fp32 kernels put row tiles (64 rows each, at most one ragged tile per expert) and, for the weight
  // gradients, 64-wide tiles of d or f on grid dimensions y / z, which hold 65535 blocks
  if (dtype == MOE_F32 && ((long long)(cap + 63) / 64 + e_cnt > 65535 || (d > f ? d : f) / 64 + 1 > 65535)) return MOE_EUNSUPPORTED;
  return MOE_OK;
}

}  // namespace

int device_cu_count() {
  static int cached[64];
  static std::once_flag once;
  std::call_once(once, [] { for (int& c : cached) c = 0; });
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// ---------------------------------------------------------------- profiling state
namespace {
struct ProfLog {
  bool on = false;
  bool made = false;
  int used = 0;
  hipEvent_t start[MOE_PROFILE_MAX_EVENTS];
  hipEvent_t stop[MOE_PROFILE_MAX_EVENTS];
  int kernel[MOE_PROFILE_MAX_EVENTS];
};
ProfLog g_prof;
}  // namespace

ProfScope::ProfScope(int kernel, hipStream_t stream) : slot(-1), s(stream) {
  if (!g_prof.on || g_prof.used >= MOE_PROFILE_MAX_EVENTS) return;
  slot = g_prof.used++;
  g_prof.kernel[slot] = kernel;
  (void)hipEventRecord(g_prof.start[slot], s);
}
ProfScope::~ProfScope() {
  if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], s);
}

extern "C" {

int moe_profile_enable(int on) {
  if (on && !g_prof.made) {
    for (int i = 0; i < MOE_PROFILE_MAX_EVENTS; ++i)
      if (hipEventCreate(&g_prof.start[i]) != hipSuccess || hipEventCreate(&g_prof.stop[i]) != hipSuccess)
        return MOE_EHIP;
    g_prof.made = true;
  }
  if (on) g_prof.used = 0;
  g_prof.on = on != 0;
  return MOE_OK;
}

int moe_profile_read(int kernel, double* total_ms, int* launches) {
  if (kernel < 0 || kernel >= MOE_K_COUNT || !total_ms || !launches) return MOE_EINVAL;
  double sum = 0.0;
  int n = 0;
  for (int i = 0; i < g_prof.used; ++i) {
    if (g_prof.kernel[i] != kernel) continue;
    if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return MOE_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess) return MOE_EHIP;
    sum += ms;
    ++n;
  }
  *total_ms = sum;
  *launches = n;
  return MOE_OK;
}

int moe_profile_stats(int kernel, double* min_ms, double* median_ms) {
  if (kernel < 0 || kernel >= MOE_K_COUNT || !min_ms || !median_ms) return MOE_EINVAL;
  std::vector<float> t;
  for (int i = 0; i < g_prof.used; ++i) {
    if (g_prof.kernel[i] != kernel) continue;
    if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return MOE_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess) return MOE_EHIP;
    t.push_back(ms);
  }
  std::sort(t.begin(), t.end());
  *min_ms = t.empty() ? 0.0 : t.front();
  *median_ms = t.empty() ? 0.0 : (t.size() % 2 ? t[t.size() / 2] : 0.5 * (t[t.size() / 2 - 1] + t[t.size() / 2]));
  return MOE_OK;
}

int moe_probe_mfma_bf16(float* sink, size_t sink_bytes, int iters, int random_operands, double* flop,
                        moe_stream_t stream) {
  if (!sink || iters <= 0 || iters > (1 << 22)) return MOE_EINVAL;
  const int cus = device_cu_count();
  if (sink_bytes < (size_t)cus * 256 * sizeof(float)) return MOE_EWORKSPACE;
  int rc = launch_probe_mfma(sink, iters, random_operands ? 1 : 0, (hipStream_t)stream);
  if (rc == MOE_OK && flop) *flop = (double)cus * 4.0 * (double)iters * 16.0 * 32768.0;
  return rc;
}

int moe_probe_mfma_fed_bf16(float* sink, size_t sink_bytes, int iters, int feed, double* flop, moe_stream_t stream) {
  if (!sink || iters <= 0 || iters > (1 << 22) || (feed != 1 && feed != 2)) return MOE_EINVAL;
  const int cus = device_cu_count();
  if (sink_bytes < (size_t)cus * 256 * sizeof(float)) return MOE_EWORKSPACE;
  int rc = launch_probe_mfma_fed(sink, iters, feed, (hipStream_t)stream);
  if (rc == MOE_OK && flop) *flop = (double)cus * 4.0 * (double)iters * 16.0 * 32768.0;
  return rc;
}

int moe_probe_stream(const void* src, void* dst, size_t bytes, int writes, void* sink, moe_stream_t stream) {
  if (writes < -1 || writes > 3 || (bytes & 15)) return MOE_EINVAL;
  if ((writes != 0 && (!src || misaligned(src, 16))) || (writes >= 0 && (!dst || misaligned(dst, 16))) ||
      (writes < 0 && (!sink || misaligned(sink, 4))))
    return MOE_EINVAL;
  if (bytes / 16 / 256 >= (1ull << 31)) return MOE_EUNSUPPORTED;
  return launch_probe_stream(src, dst, bytes, writes, (uint32_t*)sink, (hipStream_t)stream);
}

int moe_probe_copy(const void* src, void* dst, size_t bytes, moe_stream_t stream) {
  if (!src || !dst || (bytes & 15) || misaligned(src, 16) || misaligned(dst, 16)) return MOE_EINVAL;
  if (bytes / 16 / 256 >= (1ull << 31)) return MOE_EUNSUPPORTED;
  return launch_probe_copy(src, dst, bytes, (hipStream_t)stream);
}

const char* moe_error_string(int code) {
  switch (code) {
    case MOE_OK: return "ok";
    case MOE_EINVAL: return "invalid argument";
    case MOE_EUNSUPPORTED: return "unsupported shape or size";
    case MOE_EWORKSPACE: return "workspace missing, misaligned or too small";
    case MOE_EHIP: return "HIP launch failed";
    default: return "unknown error code";
  }
}

size_t moe_workspace_bytes(int which, int dtype, int T, int k, int d, int f, int e_cnt, int cap) {
  if (T < 0 || k < 0 || f < 0 || e_cnt < 0 || cap < 0) return 256;
  switch (which) {
    case MOE_WS_DISPATCH: return align256(plan_ws_bytes(T, k, e_cnt));
    case MOE_WS_EXPERT_FWD:   // a [cap,f] (+ h1, h3 when the caller does not keep them, fp32 path)
      return align256((dtype == MOE_F32 ? 3 : 1) * (size_t)cap * f * esize(dtype)) + 256;
    case MOE_WS_EXPERT_BWD:   // a, dH1, dH3 [cap,f]; bf16 adds scheduler words and the weight-gradient partial tiles
      return align256(3 * (size_t)cap * f * esize(dtype)) + (dtype == MOE_BF16 && d > 0 ? expert_bwd_extra_ws_bytes(d, f) : 256);
    case MOE_WS_ROUTER:       // e_cnt carries E
      if (d <= 0 || e_cnt <= 0) return 256;
      return router_ws_bytes(dtype, T, d, e_cnt);
    default: return 256;
  }
}

namespace {
int shape_check_router(int dtype, int T, int d, int E) {
  if (bad_dtype(dtype) || T < 0 || d <= 0 || E <= 0) return MOE_EINVAL;
  if (E > MOE_MAX_EXPERTS) return MOE_EUNSUPPORTED;
  if (dtype == MOE_BF16 && d % 8) return MOE_EUNSUPPORTED;
  // (row tiles of 64 tokens sit on grid dimension y of the plain kernels: fewer than 65536 of them)
  if ((long long)T * (d > E ? d : E) >= (1ll << 40) || T >= (1 << 22)) return MOE_EUNSUPPORTED;
  if ((long long)d * 256 >= (1ll << 31) || (long long)d * E >= (1ll << 31)) return MOE_EUNSUPPORTED;
  return MOE_OK;
}
}  // namespace

int moe_router_fwd(const void* x, const void* wr, int dtype, int T, int d, int E, float* logits, void* ws,
                   size_t ws_bytes, moe_stream_t stream) {
  int rc = shape_check_router(dtype, T, d, E);
  if (rc) return rc;
  if (!wr || (T > 0 && (!x || !logits))) return MOE_EINVAL;
  if (misaligned(x, 16) || misaligned(wr, 16) || misaligned(logits, 16)) return MOE_EINVAL;
  if (!ws || misaligned(ws, 256) || ws_bytes < router_ws_bytes(dtype, T, d, E)) return MOE_EWORKSPACE;
  return launch_router_fwd(x, wr, dtype, T, d, E, logits, ws, (hipStream_t)stream);
}

int moe_combine_bwd(const void* dy, const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                    const float* topk_w, void* d_o, float* dgate, moe_stream_t stream) {
  if (bad_dtype(dtype) || T < 0 || d <= 0 || k <= 0) return MOE_EINVAL;
  if (k > MOE_MAX_TOPK) return MOE_EUNSUPPORTED;
  if (dtype == MOE_BF16 ? d % 8 : d % 4) return MOE_EUNSUPPORTED;
  if (T > 0 && (!dy || !o || !d_o || !inv || !topk_w || !dgate)) return MOE_EINVAL;
  if (misaligned(dy, 16) || misaligned(o, 16) || misaligned(d_o, 16)) return MOE_EINVAL;
  return launch_combine_bwd(dy, o, dtype, T, d, k, inv, topk_w, d_o, dgate, (hipStream_t)stream);
}

int moe_gate_bwd(const float* logits, const int32_t* topk_idx, const float* dgate, int T, int E, int k,
                 int gate_mode, float* dlogits, moe_stream_t stream) {
  if (T < 0 || E <= 0 || k <= 0 || k > E) return MOE_EINVAL;
  if (gate_mode != MOE_GATE_SOFTMAX_RENORM && gate_mode != MOE_GATE_SIGMOID_RENORM && gate_mode != MOE_GATE_SOFTMAX)
    return MOE_EINVAL;
  if (E > MOE_MAX_EXPERTS || k > MOE_MAX_TOPK) return MOE_EUNSUPPORTED;
  if ((long long)T * E >= (1ll << 40)) return MOE_EUNSUPPORTED;
  if (T > 0 && (!logits || !topk_idx || !dgate || !dlogits)) return MOE_EINVAL;
  return launch_gate_bwd(logits, topk_idx, dgate, T, E, k, gate_mode, dlogits, (hipStream_t)stream);
}

int moe_router_bwd(const void* x, const void* wr, const float* dlogits, int dtype, int T, int d, int E,
                   void* dwr, int dwr_accumulate, void* dx, int dx_accumulate, void* ws, size_t ws_bytes,
                   moe_stream_t stream) {
  int rc = shape_check_router(dtype, T, d, E);
  if (rc) return rc;
  if ((dwr_accumulate != 0 && dwr_accumulate != 1) || (dx_accumulate != 0 && dx_accumulate != 1)) return MOE_EINVAL;
  if (!wr || (T > 0 && (!x || !dlogits))) return MOE_EINVAL;
  if (misaligned(x, 16) || misaligned(wr, 16) || misaligned(dlogits, 16) || misaligned(dwr, 16) || misaligned(dx, 16))
    return MOE_EINVAL;
  if (!ws || misaligned(ws, 256) || ws_bytes < router_ws_bytes(dtype, T, d, E)) return MOE_EWORKSPACE;
  return launch_router_bwd(x, wr, dlogits, dtype, T, d, E, dwr, dwr_accumulate, dx, dx_accumulate, ws,
                           (hipStream_t)stream);
}

int moe_route(const float* logits, int T, int E, int k, int gate_mode, int e_lo, int e_cnt,
              int32_t* topk_idx, float* topk_w, int32_t* counts, moe_stream_t stream) {
  if (T < 0 || E <= 0 || k <= 0 || k > E || e_lo < 0 || e_cnt < 0 || e_lo + (long long)e_cnt > E) return MOE_EINVAL;
  if (gate_mode != MOE_GATE_SOFTMAX_RENORM && gate_mode != MOE_GATE_SIGMOID_RENORM && gate_mode != MOE_GATE_SOFTMAX)
    return MOE_EINVAL;
  if (E > MOE_MAX_EXPERTS || e_cnt > MOE_MAX_LOCAL || k > MOE_MAX_TOPK) return MOE_EUNSUPPORTED;
  if ((long long)T * k >= (1ll << 31) || (long long)T * E >= (1ll << 40)) return MOE_EUNSUPPORTED;
  if (e_cnt > 0 && !counts) return MOE_EINVAL;
  if (T > 0 && (!logits || !topk_idx || !topk_w)) return MOE_EINVAL;
  return launch_route(logits, T, E, k, gate_mode, e_lo, e_cnt, topk_idx, topk_w, counts, (hipStream_t)stream);
}

int moe_dispatch(const void* x, int dtype, int T, int d, int k, const int32_t* topk_idx,
                 const float* row_scale, int e_lo, int e_cnt, int32_t* offsets, int32_t* perm,
                 int32_t* inv, int reuse_plan, void* xp, int cap, void* ws, size_t ws_bytes,
                 moe_stream_t stream) {
  if (bad_dtype(dtype) || T < 0 || d <= 0 || k <= 0 || e_lo < 0 || e_cnt < 0 || cap < 0) return MOE_EINVAL;
  if (k > MOE_MAX_TOPK || e_cnt > MOE_MAX_LOCAL) return MOE_EUNSUPPORTED;
  if ((long long)T * k >= (1ll << 31)) return MOE_EUNSUPPORTED;
  if (dtype == MOE_BF16 ? d % 8 : d % 4) return MOE_EUNSUPPORTED;
  if ((long long)T * ((d / (dtype == MOE_BF16 ? 8 : 4) + 127) / 128) >= (1ll << 31)) return MOE_EUNSUPPORTED;   // mover grid
  if (!offsets) return MOE_EINVAL;
  if (T > 0 && (!x || !inv)) return MOE_EINVAL;
  if (cap > 0 && (!xp || !perm)) return MOE_EINVAL;
  if (misaligned(x, 16) || misaligned(xp, 16)) return MOE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (!reuse_plan) {
    if (T > 0 && !topk_idx) return MOE_EINVAL;
    if (!ws || misaligned(ws, 256) || ws_bytes < plan_ws_bytes(T, k, e_cnt)) return MOE_EWORKSPACE;
    int rc = launch_plan(topk_idx, T, k, e_lo, e_cnt, offsets, perm, inv, cap, ws, nullptr, s);
    if (rc) return rc;
  }
  return launch_dispatch_rows(x, dtype, T, d, k, inv, row_scale, xp, s);
}

int moe_dispatch_static(const void* x, int dtype, int T, int d, int k, const int32_t* topk_idx,
                        const float* row_scale, int e_lo, int e_cnt, int32_t* offsets, int32_t* perm,
                        int32_t* inv, void* xp, int cap, int32_t* status, moe_stream_t stream) {
  if (bad_dtype(dtype) || T < 0 || d <= 0 || k <= 0 || e_lo < 0 || e_cnt < 0 || cap < 0) return MOE_EINVAL;
  if (k > MOE_MAX_TOPK || e_cnt > MOE_MAX_LOCAL) return MOE_EUNSUPPORTED;
  if ((long long)T * k >= (1ll << 31)) return MOE_EUNSUPPORTED;
  if (dtype == MOE_BF16 ? d % 8 : d % 4) return MOE_EUNSUPPORTED;
  if ((long long)T * ((d / (dtype == MOE_BF16 ? 8 : 4) + 127) / 128) >= (1ll << 31)) return MOE_EUNSUPPORTED;   // mover grid
  if (!offsets) return MOE_EINVAL;
  if (T > 0 && (!x || !inv || !topk_idx)) return MOE_EINVAL;
  if (cap > 0 && (!xp || !perm)) return MOE_EINVAL;
  if (misaligned(x, 16) || misaligned(xp, 16)) return MOE_EINVAL;
  // the plan tables of this call must fit the built-in scratch
  if (plan_ws_bytes(T, k, e_cnt) > (size_t)MOE_STATIC_PLAN_BYTES) return MOE_EWORKSPACE;
  void* ws = nullptr;
  int rc = plan_static_scratch(&ws);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  if ((rc = launch_plan(topk_idx, T, k, e_lo, e_cnt, offsets, perm, inv, cap, ws, status, s))) return rc;
  return launch_dispatch_rows(x, dtype, T, d, k, inv, row_scale, xp, s);
}

int moe_expert_fwd(const void* xp, int dtype, int cap, int d, int f, int e_cnt,
                   const int32_t* offsets, const void* w1, const void* w3, const void* w2,
                   void* h1, void* h3, void* a_out, void* o, void* ws, size_t ws_bytes, moe_stream_t stream) {
  int rc = shape_check_expert(dtype, cap, d, f, e_cnt);
  if (rc) return rc;
  if (!offsets) return MOE_EINVAL;
  if ((h1 == nullptr) != (h3 == nullptr)) return MOE_EINVAL;
  if (e_cnt > 0 && (!w1 || !w3 || !w2)) return MOE_EINVAL;
  if (cap > 0 && (!xp || !o)) return MOE_EINVAL;
  if (misaligned(xp, 16) || misaligned(o, 16) || misaligned(h1, 16) || misaligned(h3, 16) || misaligned(a_out, 16) ||
      misaligned(w1, 16) || misaligned(w3, 16) || misaligned(w2, 16))
    return MOE_EINVAL;
  if (!ws || misaligned(ws, 256) || ws_bytes < moe_workspace_bytes(MOE_WS_EXPERT_FWD, dtype, 0, 0, d, f, e_cnt, cap))
    return MOE_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  if (dtype == MOE_BF16)
    return launch_expert_fwd_bf16(xp, cap, d, f, e_cnt, offsets, w1, w3, w2, h1, h3, a_out, o, ws, s);
  float* a = a_out ? (float*)a_out : (float*)ws;
  float* t1 = h1 ? (float*)h1 : (float*)ws + (size_t)cap * f;
  float* t3 = h3 ? (float*)h3 : (float*)ws + 2 * (size_t)cap * f;
  return launch_expert_fwd_f32((const float*)xp, cap, d, f, e_cnt, offsets, (const float*)w1, (const float*)w3,
                               (const float*)w2, t1, t3, (float*)o, a, s);
}

int moe_expert_bwd(const void* xp, const void* h1, const void* h3, const void* a_in, const void* d_o, int dtype,
                   int cap, int d, int f, int e_cnt, const int32_t* offsets, const void* w1,
                   const void* w3, const void* w2, void* dxp, void* dw1, void* dw3, void* dw2,
                   int accumulate, void* ws, size_t ws_bytes, moe_stream_t stream) {
  int rc = shape_check_expert(dtype, cap, d, f, e_cnt);
  if (rc) return rc;
  if (!offsets || (accumulate != 0 && accumulate != 1)) return MOE_EINVAL;
  if (e_cnt > 0 && (!w1 || !w3 || !w2 || !dw1 || !dw3 || !dw2)) return MOE_EINVAL;
  if (cap > 0 && (!xp || !h1 || !h3 || !d_o || !dxp)) return MOE_EINVAL;
  if (misaligned(xp, 16) || misaligned(h1, 16) || misaligned(h3, 16) || misaligned(d_o, 16) || misaligned(a_in, 16) ||
      misaligned(dxp, 16) || misaligned(w1, 16) || misaligned(w3, 16) || misaligned(w2, 16) ||
      misaligned(dw1, 16) || misaligned(dw3, 16) || misaligned(dw2, 16))
    return MOE_EINVAL;
  if (!ws || misaligned(ws, 256) || ws_bytes < moe_workspace_bytes(MOE_WS_EXPERT_BWD, dtype, 0, 0, d, f, e_cnt, cap))
    return MOE_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  if (dtype == MOE_BF16)
    return launch_expert_bwd_bf16(xp, h1, h3, a_in, d_o, cap, d, f, e_cnt, offsets, w1, w3, w2, dxp, dw1, dw3, dw2,
                                  accumulate, ws, s);
  return launch_expert_bwd_f32((const float*)xp, (const float*)h1, (const float*)h3, (const float*)a_in, (const float*)d_o, cap, d, f,
                               e_cnt, offsets, (const float*)w1, (const float*)w3, (const float*)w2, (float*)dxp,
                               (float*)dw1, (float*)dw3, (float*)dw2, accumulate, (float*)ws, s);
}

int moe_combine(const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                const float* topk_w, void* y, moe_stream_t stream) {
  if (bad_dtype(dtype) || T < 0 || d <= 0 || k <= 0) return MOE_EINVAL;
  if (k > MOE_MAX_TOPK) return MOE_EUNSUPPORTED;
  if (dtype == MOE_BF16 ? d % 8 : d % 4) return MOE_EUNSUPPORTED;
  if ((long long)T * ((d / (dtype == MOE_BF16 ? 8 : 4) + 127) / 128) >= (1ll << 31)) return MOE_EUNSUPPORTED;   // mover grid
  if (T > 0 && (!o || !inv || !y)) return MOE_EINVAL;
  if (misaligned(o, 16) || misaligned(y, 16)) return MOE_EINVAL;
  return launch_combine_rows(o, dtype, T, d, k, inv, topk_w, y, (hipStream_t)stream);
}

}  // extern "C"
