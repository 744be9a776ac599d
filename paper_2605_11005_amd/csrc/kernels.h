// Internal launch functions behind the C ABI (one per kernel family).  Arguments have been
// validated by api.hip; every function only enqueues work on `s` and returns a MOE_* code.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "../../include/moe.h"

int launch_route(const float* logits, int T, int E, int k, int gate_mode, int e_lo, int e_cnt,
                 int32_t* topk_idx, float* topk_w, int32_t* counts, hipStream_t s);

size_t plan_ws_bytes(int T, int k, int e_cnt);
// status_out: where the overflow status word goes (NULL: the first word of ws)
int launch_plan(const int32_t* topk_idx, int T, int k, int e_lo, int e_cnt, int32_t* offsets,
                int32_t* perm, int32_t* inv, int cap, void* ws, int32_t* status_out, hipStream_t s);
// device address of this GPU's built-in plan scratch (MOE_STATIC_PLAN_BYTES bytes); looks it up on first use
int plan_static_scratch(void** ptr);

int launch_dispatch_rows(const void* x, int dtype, int T, int d, int k, const int32_t* inv,
                         const float* row_scale, void* xp, hipStream_t s);
int launch_combine_rows(const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                        const float* topk_w, void* y, hipStream_t s);

int launch_expert_fwd_f32(const float* xp, int cap, int d, int f, int e_cnt, const int32_t* offsets,
                          const float* w1, const float* w3, const float* w2, float* h1, float* h3,
                          float* o, float* a_ws, hipStream_t s);
int launch_expert_bwd_f32(const float* xp, const float* h1, const float* h3, const float* a_in, const float* d_o, int cap,
                          int d, int f, int e_cnt, const int32_t* offsets, const float* w1,
                          const float* w3, const float* w2, float* dxp, float* dw1, float* dw3,
                          float* dw2, int accumulate, float* ws, hipStream_t s);

int launch_expert_fwd_bf16(const void* xp, int cap, int d, int f, int e_cnt, const int32_t* offsets,
                           const void* w1, const void* w3, const void* w2, void* h1, void* h3, void* a_out, void* o,
                           void* a_ws, hipStream_t s);
int launch_expert_bwd_bf16(const void* xp, const void* h1, const void* h3, const void* a_in, const void* d_o, int cap,
                           int d, int f, int e_cnt, const int32_t* offsets, const void* w1,
                           const void* w3, const void* w2, void* dxp, void* dw1, void* dw3, void* dw2,
                           int accumulate, void* ws, hipStream_t s);

// trainable router (router.hip; the matrix-core variants live in expert_bf16.hip)
size_t router_ws_bytes(int dtype, int T, int d, int E);
int launch_router_fwd(const void* x, const void* wr, int dtype, int T, int d, int E, float* logits, void* ws,
                      hipStream_t s);
int launch_combine_bwd(const void* dy, const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                       const float* topk_w, void* d_o, float* dgate, hipStream_t s);
int launch_gate_bwd(const float* logits, const int32_t* topk_idx, const float* dgate, int T, int E, int k,
                    int gate_mode, float* dlogits, hipStream_t s);
int launch_router_bwd(const void* x, const void* wr, const float* dlogits, int dtype, int T, int d, int E, void* dwr,
                      int dwr_acc, void* dx, int dx_acc, void* ws, hipStream_t s);
int router_dw_splits(int T, int d, int E);
int router_fwd_splits(int T, int d, int E);
int launch_router_fwd_bf16(const void* x, const void* wr, int T, int d, int E, float* logits, float* partials,
                           int splits, int32_t* sched, hipStream_t s);
int launch_router_dw_bf16(const void* x, const void* dl_bf16, int T, int d, int E, float* partials, int splits,
                          int32_t* sched, hipStream_t s);
int launch_router_dx_bf16(const void* dl_bf16, const void* wr, int T, int d, int E, void* dx, int accumulate,
                          int32_t* sched, hipStream_t s);
int launch_zero_words(int32_t* p, int n, hipStream_t s);

// bytes that launch_expert_bwd_bf16 uses after the three [cap,f] activation buffers
size_t expert_bwd_extra_ws_bytes(int d, int f);
size_t wgrad_split_bytes(int d, int f);

int launch_probe_mfma(float* sink, int iters, int random_operands, hipStream_t s);
int launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
int launch_probe_mfma_fed(float* sink, int iters, int feed, hipStream_t s);
int launch_probe_stream(const void* src, void* dst, size_t bytes, int writes, uint32_t* sink, hipStream_t s);

int device_cu_count();

// Per-kernel timing (moe_profile_*): brackets a launch with events when profiling is on.
struct ProfScope {
  int slot;
  hipStream_t s;
  ProfScope(int kernel, hipStream_t stream);
  ~ProfScope();
};
