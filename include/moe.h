/*
 * moe.h -- C ABI of the MI355X (gfx950) MoE expert-layer library.
 *
 * One FFN-group GPU's share of a Mixture-of-Experts layer: top-k gating, the shuffle of
 * tokens from micro-batch order into expert order, the SwiGLU expert FFNs as grouped
 * GEMMs (forward and backward), and the gate-weighted reduction back to token order.
 *
 * Notation (the paper's symbol table in brackets): T tokens [b*s], d hidden size [H],
 * E experts, k top-k, f expert hidden size [D_e].  This GPU holds the contiguous expert
 * slice [e_lo, e_lo+e_cnt) (expert parallelism, background section on distributed
 * training).  R = number of (token, slot) pairs routed to a local expert.
 *
 * Conventions for every entry point
 *   - All pointers are DEVICE pointers unless marked "host".  All matrices are row-major
 *     and densely packed.  Integer scalars are host values.
 *   - dtype is MOE_F32 (float) or MOE_BF16 (bfloat16 storage, fp32 accumulation,
 *     round-to-nearest-even stores).  It is the type of x/xp/h/o/y and of the weights.
 *   - The caller owns every buffer.  The library allocates no device memory, keeps no
 *     pointer past the call and never synchronises with the host: each call only enqueues
 *     kernels on `stream` (a hipStream_t; NULL = the default stream).  Row counts stay on
 *     the device (offsets[e_cnt] = R), so a whole layer can be enqueued without a sync.
 *   - Return value: MOE_OK or an error code.  Arguments are validated on the host before
 *     anything is launched; on error nothing has been enqueued.  No exception or abort
 *     crosses this boundary.  Inputs must be finite (NaN/Inf logits: unspecified
 *     selection, but no out-of-bounds access).
 *   - T == 0 is legal and a no-op (plan outputs are still written: all offsets zero).
 */
#ifndef MOE_MI355X_H
#define MOE_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void* moe_stream_t; /* hipStream_t */

enum { MOE_OK = 0, MOE_EINVAL = 1, MOE_EUNSUPPORTED = 2, MOE_EWORKSPACE = 3, MOE_EHIP = 4 };
enum { MOE_F32 = 0, MOE_BF16 = 1 };
enum { MOE_GATE_SOFTMAX_RENORM = 0, MOE_GATE_SIGMOID_RENORM = 1, MOE_GATE_SOFTMAX = 2 };
enum { MOE_WS_DISPATCH = 0, MOE_WS_EXPERT_FWD = 1, MOE_WS_EXPERT_BWD = 2, MOE_WS_ROUTER = 3 };

/* Limits checked by the entry points (MOE_EUNSUPPORTED beyond them). */
#define MOE_MAX_EXPERTS 1024 /* E */
#define MOE_MAX_LOCAL 1024   /* e_cnt */
#define MOE_MAX_TOPK 64      /* k */

/*
 * moe_route -- top-k gating (MoE background section: a gate network selects the top-k
 * experts with the highest probability scores).
 *
 *   logits  [T,E] float     router outputs (the router GEMM itself is the caller's)
 *   topk_idx[T,k] int32     out: global expert ids; slot j = j-th best.  Ranking is on the
 *                           raw fp32 logits, descending; equal logits (+0 == -0) -> the
 *                           lower expert id first.
 *   topk_w  [T,k] float     out: gate weights.  SOFTMAX_RENORM: softmax over all E,
 *                           renormalised over the k selected; SIGMOID_RENORM: logistic
 *                           scores renormalised over the k selected; SOFTMAX: softmax over
 *                           all E, not renormalised.
 *   counts  [e_cnt] int32   out: number of slots routed to each local expert.
 * Errors: EINVAL for NULL pointers, T<0, E<=0, k<=0, k>E, slice outside [0,E), unknown
 * gate_mode; EUNSUPPORTED beyond the limits above.
 */
int moe_route(const float* logits, int T, int E, int k, int gate_mode, int e_lo, int e_cnt,
              int32_t* topk_idx, float* topk_w, int32_t* counts, moe_stream_t stream);

/*
 * moe_dispatch -- shuffle tokens from micro-batch order to expert order (introduction:
 * tokens are dispatched from the micro-batch ranking to the expert ranking; the paper's
 * resource-allocation section counts 2*S*k*H bytes of bf16 per direction for it).
 *
 * Plan (reuse_plan == 0): from topk_idx build
 *   offsets [e_cnt+1] int32  out: exclusive prefix sum of the local counts; offsets[e_cnt]=R
 *   perm    [cap]     int32  out: perm[r] = flat slot s = t*k + j held by row r; rows are
 *                            sorted by (local expert, s) -- a stable counting sort, so the
 *                            result is unique and reproducible.  Entries [R,cap) untouched.
 *   inv     [T,k]     int32  out: row of slot (t,j), or -1 if its expert is not local.
 * With reuse_plan == 1 the three arrays are inputs (as written by an earlier call) and
 * topk_idx may be NULL.
 * Row move: xp[inv[t,j], :] = x[t, :] * (row_scale ? row_scale[t,j] : 1) for every local
 * slot.  Rows [R,cap) of xp are left untouched.  The scaled form is the backward of
 * moe_combine with respect to its input (d_o = gate * dy); the product is formed in fp32
 * and rounded once.
 *
 *   x        [T,d] dtype     tokens (or dy)
 *   row_scale[T,k] float     NULL or per-slot factor
 *   xp       [cap,d] dtype   out
 *   cap                      rows available in xp/perm.  cap >= R is the caller's duty
 *                            (T*min(k,e_cnt) always suffices).  If R > cap, rows >= cap are
 *                            dropped (their inv is -1), offsets are clamped to cap and the
 *                            int32 status word at the start of ws is set to 1 (else 0).
 *   ws, ws_bytes             device scratch of at least
 *                            moe_workspace_bytes(MOE_WS_DISPATCH, ...) bytes, 256-byte
 *                            aligned; only used when reuse_plan == 0.
 * Errors: EINVAL (NULL, negative sizes, k>MOE_MAX_TOPK, bad slice, unknown dtype),
 * EUNSUPPORTED (bf16 with d % 8 != 0, fp32 with d % 4 != 0), EWORKSPACE.
 */
int moe_dispatch(const void* x, int dtype, int T, int d, int k, const int32_t* topk_idx,
                 const float* row_scale, int e_lo, int e_cnt, int32_t* offsets, int32_t* perm,
                 int32_t* inv, int reuse_plan, void* xp, int cap, void* ws, size_t ws_bytes,
                 moe_stream_t stream);

/*
 * moe_dispatch_static -- moe_dispatch (plan + row move, reuse_plan == 0) for callers that cannot
 * allocate device memory or pass a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The plan's scratch (its per-chunk histogram table and the
 * expert bases) lives in a MOE_STATIC_PLAN_BYTES array inside the library's code object; each GPU
 * that runs the library holds its own copy until the process ends.  The call allocates nothing
 * and frees nothing.  Outputs are bit-identical to moe_dispatch's.
 *   arguments as moe_dispatch, without reuse_plan / ws / ws_bytes, plus
 *   status   int32 (device) out, may be NULL: 1 if R > cap (rows dropped as in moe_dispatch), else 0.
 * Limit: the plan tables must fit the array, 256 + 4 (ceil(T k / 512) e_cnt + e_cnt + 1) <=
 * MOE_STATIC_PLAN_BYTES (at e_cnt = 32 that is T k <= 16.7 million slots); beyond it the call
 * returns MOE_EWORKSPACE and enqueues nothing.  Other errors as moe_dispatch.
 * The array is shared by every call on a GPU and keeps the last call's contents (each call
 * overwrites what it reads, nothing needs clearing): calls that overlap on one GPU, on different
 * streams or from different threads, race; serialise them.  The first call on a device looks up
 * the array's device address (no allocation); make it before a graph capture starts.
 */
#define MOE_STATIC_PLAN_BYTES (4 << 20)
int moe_dispatch_static(const void* x, int dtype, int T, int d, int k, const int32_t* topk_idx,
                        const float* row_scale, int e_lo, int e_cnt, int32_t* offsets, int32_t* perm,
                        int32_t* inv, void* xp, int cap, int32_t* status, moe_stream_t stream);

/*
 * moe_expert_fwd -- the expert FFNs as grouped GEMMs over expert-contiguous rows
 * (resource-allocation section: after gating, GroupGEMMs over the k*S routed tokens).
 * For each local expert e and its rows [offsets[e], offsets[e+1]):
 *     h1 = xp W1[e];  h3 = xp W3[e];  a = silu(h1) * h3;  o = a W2[e]
 * with silu(z) = z / (1 + exp(-z)).
 *
 *   xp [cap,d]; w1,w3 [e_cnt,d,f]; w2 [e_cnt,f,d] (local slice: index 0 = expert e_lo)
 *   h1,h3 [cap,f]  out, saved for the backward pass; both NULL = forward only
 *   a  [cap,f]     out, may be NULL: the activation silu(h1) * h3 as the down projection consumed it
 *                  (rounded to dtype).  A caller that keeps it and hands it to moe_expert_bwd saves that
 *                  call one [cap,f] store; with NULL it goes to ws and the backward recomputes it.
 *   o  [cap,d]     out.  Rows >= R of every output are left untouched.
 *   ws             device scratch (holds a [cap,f] and the tile-scheduler counters),
 *                  moe_workspace_bytes(MOE_WS_EXPERT_FWD, ...) bytes, 256-byte aligned
 * bf16 requires d % 64 == 0 and f % 64 == 0; fp32 requires d % 4 == 0 and f % 4 == 0
 * (EUNSUPPORTED otherwise).  offsets must be non-decreasing with offsets[e_cnt] <= cap.
 */
int moe_expert_fwd(const void* xp, int dtype, int cap, int d, int f, int e_cnt,
                   const int32_t* offsets, const void* w1, const void* w3, const void* w2,
                   void* h1, void* h3, void* a, void* o, void* ws, size_t ws_bytes, moe_stream_t stream);

/*
 * moe_expert_bwd -- backward of moe_expert_fwd (AF-Pipe section: FFN workers run backward
 * passes and send hidden-state gradients back).  Per expert e, on its rows:
 *     dA  = d_o W2[e]^T                      dW2[e] = a^T d_o
 *     dH1 = dA * h3 * silu'(h1)              dH3    = dA * silu(h1)
 *     dW1[e] = xp^T dH1                      dW3[e] = xp^T dH3
 *     dxp = dH1 W1[e]^T + dH3 W3[e]^T
 * with silu'(z) = s(z) (1 + z (1 - s(z))), s the logistic function.
 *
 *   xp,h1,h3 as saved by the forward; d_o [cap,d] gradient w.r.t. o
 *   a [cap,f]     the forward's activation output, or NULL.  With NULL it is recomputed from the saved
 *                 (rounded) h1, h3 into ws, which differs from the forward's value by one rounding of
 *                 h1 and h3; with the forward's copy dW2 is the gradient of exactly what the forward
 *                 multiplied by W2, and the call stores one [cap,f] matrix less.
 *   dxp [cap,d] out; dw1,dw3 [e_cnt,d,f], dw2 [e_cnt,f,d] out (dtype = weight dtype)
 *   accumulate    0: dw* are overwritten (an expert without rows gets zeros);
 *                 1: the new gradient is added to the existing contents.
 *   ws            device scratch (a, dH1, dH3 [cap,f], the tile-scheduler counters and, for bf16,
 *                 fp32 partial tiles for the weight gradients of experts with far more rows than
 *                 the others, which are accumulated in pieces -- at most 512 MB),
 *                 moe_workspace_bytes(MOE_WS_EXPERT_BWD, ...) bytes, 256-byte aligned.
 * Results are bit-reproducible from run to run (every sum has a fixed order).
 * Same shape restrictions as the forward.
 */
int moe_expert_bwd(const void* xp, const void* h1, const void* h3, const void* a, const void* d_o, int dtype,
                   int cap, int d, int f, int e_cnt, const int32_t* offsets, const void* w1,
                   const void* w3, const void* w2, void* dxp, void* dw1, void* dw3, void* dw2,
                   int accumulate, void* ws, size_t ws_bytes, moe_stream_t stream);

/*
 * moe_combine -- gate-weighted reduction back to token order (MoE background section:
 * the outputs of the active experts are reduced by a weighted sum).
 *     y[t,:] = sum over j with inv[t,j] >= 0, ascending j, of topk_w[t,j] * o[inv[t,j], :]
 * accumulated in fp32 and rounded once; tokens without a local slot get zeros.  With
 * topk_w == NULL every weight is 1 (the backward of the unscaled dispatch: dx from dxp).
 *   o [rows,d] dtype; inv [T,k]; topk_w [T,k] float or NULL; y [T,d] dtype out.
 * Every inv entry must be -1 or a valid row of o.
 */
int moe_combine(const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                const float* topk_w, void* y, moe_stream_t stream);

/* Scratch bytes needed by the call named by `which` (MOE_WS_*) at these sizes; 0 on
 * invalid arguments is never returned for valid ones (at least 256).  For MOE_WS_ROUTER
 * (moe_router_fwd and moe_router_bwd share one size) pass E in the e_cnt argument. */
size_t moe_workspace_bytes(int which, int dtype, int T, int k, int d, int f, int e_cnt, int cap);

/*
 * The trainable gate (MoE background section: the gate network that scores the experts is
 * trainable).  logits = x Wr, and the loss reaches Wr and x a second time through the gate
 * weights that multiply the expert outputs.  Expert selection is held fixed in the backward
 * pass (it is piecewise constant in the logits).  Order of the calls in a training step:
 *   forward : moe_router_fwd -> moe_route -> moe_dispatch -> moe_expert_fwd -> moe_combine
 *   backward: moe_combine_bwd (replaces the scaled moe_dispatch) -> moe_expert_bwd ->
 *             moe_combine(dxp, no gate) -> moe_gate_bwd -> moe_router_bwd (adds into dx)
 *
 * moe_router_fwd -- logits [T,E] float = x [T,d] Wr [d,E], fp32 accumulation.
 *   x and wr have type `dtype`; bf16 requires d % 8 == 0.  ws: moe_workspace_bytes(MOE_WS_ROUTER).
 */
int moe_router_fwd(const void* x, const void* wr, int dtype, int T, int d, int E, float* logits,
                   void* ws, size_t ws_bytes, moe_stream_t stream);

/*
 * moe_combine_bwd -- backward of moe_combine with respect to both of its inputs, in one pass
 * over dy:
 *     d_o[inv[t,j], :] = topk_w[t,j] * dy[t, :]                    (as the scaled moe_dispatch)
 *     dgate[t,j]       = < dy[t, :], o[inv[t,j], :] >               (0 where inv[t,j] == -1)
 *   dy [T,d], o [rows,d], d_o [rows,d] of type dtype; inv [T,k]; topk_w, dgate [T,k] float.
 * The dot product is accumulated in fp32 in a fixed order (reproducible run to run).  With a
 * local expert slice dgate holds this GPU's slots only; moe_gate_bwd is linear in dgate, so
 * partial results add across GPUs.
 */
int moe_combine_bwd(const void* dy, const void* o, int dtype, int T, int d, int k, const int32_t* inv,
                    const float* topk_w, void* d_o, float* dgate, moe_stream_t stream);

/*
 * moe_gate_bwd -- gradient with respect to the logits through the gate weights, selection fixed.
 * With g the gate weights of the k selected experts and c = sum_j g_j dgate_j:
 *   SOFTMAX_RENORM : dlogit_j = g_j (dgate_j - c)                 on the selected experts, else 0
 *   SIGMOID_RENORM : dlogit_j = (dgate_j - c) s_j (1 - s_j) / S   (s logistic scores, S their sum
 *                                                                  over the selection), else 0
 *   SOFTMAX        : dlogit_e = p_e ([e selected] dgate_e - c)    for all E (p softmax over all E)
 *   logits [T,E] float, topk_idx [T,k], dgate [T,k] float -> dlogits [T,E] float (every entry written).
 */
int moe_gate_bwd(const float* logits, const int32_t* topk_idx, const float* dgate, int T, int E, int k,
                 int gate_mode, float* dlogits, moe_stream_t stream);

/*
 * moe_router_bwd -- backward of moe_router_fwd:
 *     dwr [d,E] (+)= x^T dlogits          dx [T,d] (+)= dlogits Wr^T
 *   dwr, dx of type dtype; dlogits [T,E] float.  dwr_accumulate / dx_accumulate: 0 overwrite,
 *   1 add to the existing contents (dx_accumulate = 1 adds the router term to the gradient that
 *   the expert path left in dx).  Either output may be NULL to skip it.
 *   bf16: dlogits is rounded to bf16 for the matrix cores when E % 64 == 0 and d % 64 == 0
 *   (fp32 accumulation over T in fixed-size chunks, chunk sums added in fp32); other shapes
 *   take a plain fp32 path.  ws: moe_workspace_bytes(MOE_WS_ROUTER).
 */
int moe_router_bwd(const void* x, const void* wr, const float* dlogits, int dtype, int T, int d, int E,
                   void* dwr, int dwr_accumulate, void* dx, int dx_accumulate, void* ws, size_t ws_bytes,
                   moe_stream_t stream);

/*
 * Optional per-kernel timing, for benchmarks (measurement of the grouped GEMMs against the
 * MFMA roofline and of the row movers against HBM bandwidth).  Apart from per-device caches of
 * constants (CU count, the kernels' LDS opt-in attribute, the address of the built-in plan scratch)
 * this is the library's only process-wide state, and it is off by default.  While enabled, every kernel launch of the
 * entry points above is bracketed by a pair of hipEvents recorded on the call's stream
 * (a few microseconds of host work per launch; no synchronisation).
 *   moe_profile_enable(on)   on != 0: create the event pool (first time) and start recording
 *                            from an empty log; on == 0: stop recording.
 *   moe_profile_read(kernel, &total_ms, &launches)
 *                            synchronises on the recorded events of that kernel (MOE_K_*)
 *                            and returns the summed elapsed time and the launch count.
 *   moe_profile_stats(kernel, &min_ms, &median_ms)
 *                            the shortest and the median launch of that kernel in the log
 *                            (0 if it holds none); synchronises like moe_profile_read.
 * The pool holds MOE_PROFILE_MAX_EVENTS launches; later launches are not recorded.
 * Not thread-safe: enable, run and read from one host thread.
 */
enum { MOE_K_ROUTE = 0, MOE_K_PLAN = 1, MOE_K_DISPATCH = 2, MOE_K_COMBINE = 3, MOE_K_UP = 4,
       MOE_K_DOWN = 5, MOE_K_DA = 6, MOE_K_DX = 7, MOE_K_WG = 8, MOE_K_WGD = 9, MOE_K_ROUTER_FWD = 10,
       MOE_K_COMBINE_BWD = 11, MOE_K_GATE_BWD = 12, MOE_K_ROUTER_DW = 13, MOE_K_ROUTER_DX = 14,
       MOE_K_WGRAD_REDUCE = 15,   /* sum of the fp32 partial tiles of weight gradients cut along the rows */
       /* bf16 backward: GEMMs that do not depend on each other may share a launch (the second fills
        * the first one's tail): dA with dW2 when moe_expert_bwd is given the forward's a, dX with
        * dW1|dW3, each when the capacity bound gives a workgroup at most a dozen tiles of the first.
        * A shared launch is booked here and not under the single ids. */
       MOE_K_DA_WG = 16, MOE_K_DX_WGD = 17,
       MOE_K_COUNT = 18 };
#define MOE_PROFILE_MAX_EVENTS 8192
int moe_profile_enable(int on);
int moe_profile_read(int kernel, double* total_ms /* host */, int* launches /* host */);
int moe_profile_stats(int kernel, double* min_ms /* host */, double* median_ms /* host */);

/*
 * Measured ceilings, for benchmarks only (not part of the expert-layer path): the rates this
 * chip sustains under its own clock and power management, to be timed by the caller with
 * events on `stream`.
 *   moe_probe_mfma_bf16  enqueues an MFMA-only loop (32x32x16 bf16, 4 wavefronts per CU,
 *                        16 independent accumulators, no memory traffic), `iters` rounds of 16
 *                        MFMAs per wavefront; operands constant or pseudo-random (the latter
 *                        is the realistic case: switching activity lowers the sustained clock).
 *                        sink: device scratch of >= 256*4 bytes per CU; *flop (host) receives
 *                        the FLOP count of the launch.
 *   moe_probe_mfma_fed_bf16  the same loop with random operands re-read from LDS before every 16 MFMAs, at
 *                        the rate the grouped GEMM's tiling needs (8 fragments of 16 bytes per lane):
 *                        feed = 1 with 16-byte reads, feed = 2 with pairs of 8-byte transposing reads.  It
 *                        prices the operand feed under the package power limit.
 *   moe_probe_copy       enqueues a plain device copy of `bytes` (multiple of 16) bytes.
 *   moe_probe_stream     streaming kernels with the row movers' access width, for their ceilings: over
 *                        `bytes` (multiple of 16) of src, writes = -1 reads only (sink: >= 4 bytes of device
 *                        memory, never written in practice), 0 fills dst, n = 1..3 reads each 16-byte vector
 *                        once and writes it n times (dst must hold n * bytes).
 */
int moe_probe_mfma_bf16(float* sink, size_t sink_bytes, int iters, int random_operands, double* flop /* host */,
                        moe_stream_t stream);
int moe_probe_mfma_fed_bf16(float* sink, size_t sink_bytes, int iters, int feed, double* flop /* host */,
                            moe_stream_t stream);
int moe_probe_copy(const void* src, void* dst, size_t bytes, moe_stream_t stream);
int moe_probe_stream(const void* src, void* dst, size_t bytes, int writes, void* sink, moe_stream_t stream);

/* Static, human-readable text for an error code. */
const char* moe_error_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* MOE_MI355X_H */
