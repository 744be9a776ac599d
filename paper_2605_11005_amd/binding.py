"""ctypes binding of include/moe.h.  Argument marshalling only.

Every function takes torch CUDA tensors (device memory) and forwards their data pointers,
the sizes and torch's current HIP stream to the C entry point of the same name.  There is
no fallback: if libmoe_mi355x.so is missing or a call returns an error code, MoeError is
raised.
"""
from __future__ import annotations

import ctypes
import os

MOE_F32, MOE_BF16 = 0, 1
GATE_SOFTMAX_RENORM, GATE_SIGMOID_RENORM, GATE_SOFTMAX = 0, 1, 2
WS_DISPATCH, WS_EXPERT_FWD, WS_EXPERT_BWD, WS_ROUTER = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = ("moe_route", "moe_dispatch", "moe_dispatch_static", "moe_expert_fwd", "moe_expert_bwd", "moe_combine",
           "moe_router_fwd", "moe_combine_bwd", "moe_gate_bwd", "moe_router_bwd",
           "moe_profile_enable", "moe_profile_read", "moe_profile_stats", "moe_probe_mfma_bf16", "moe_probe_mfma_fed_bf16",
           "moe_probe_copy", "moe_probe_stream",
           "moe_workspace_bytes", "moe_error_string")


class MoeError(RuntimeError):
    pass


def lib_path() -> str:
    return os.path.join(_HERE, "libmoe_mi355x.so")


def load_library():
    """Load the HIP library (built by __graft_entry__.build() / csrc/build.sh)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise MoeError(f"{path} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(path)
    c_int, c_void_p, c_size_t = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.moe_route.restype = c_int
    lib.moe_route.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.moe_dispatch.restype = c_int
    lib.moe_dispatch.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_int, c_int, c_void_p,
                                 c_void_p, c_void_p, c_int, c_void_p, c_int, c_void_p, c_size_t, c_void_p]
    lib.moe_dispatch_static.restype = c_int
    lib.moe_dispatch_static.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_int, c_int, c_void_p,
                                        c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p]
    lib.moe_expert_fwd.restype = c_int
    lib.moe_expert_fwd.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p,
                                   c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.moe_expert_bwd.restype = c_int
    lib.moe_expert_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p,
                                   c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int,
                                   c_void_p, c_size_t, c_void_p]
    lib.moe_combine.restype = c_int
    lib.moe_combine.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.moe_router_fwd.restype = c_int
    lib.moe_router_fwd.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.moe_combine_bwd.restype = c_int
    lib.moe_combine_bwd.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                    c_void_p, c_void_p]
    lib.moe_gate_bwd.restype = c_int
    lib.moe_gate_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p]
    lib.moe_router_bwd.restype = c_int
    lib.moe_router_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_int, c_void_p,
                                   c_int, c_void_p, c_size_t, c_void_p]
    lib.moe_workspace_bytes.restype = c_size_t
    lib.moe_workspace_bytes.argtypes = [c_int] * 8
    lib.moe_error_string.restype = ctypes.c_char_p
    lib.moe_error_string.argtypes = [c_int]
    _LIB = lib
    return lib


def _check(rc: int, name: str):
    if rc != 0:
        raise MoeError(f"{name} failed: {load_library().moe_error_string(rc).decode()} (code {rc})")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise MoeError(f"unsupported dtype {t.dtype}")


def _need(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise MoeError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise MoeError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise MoeError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")


def moe_workspace_bytes(which, dtype, T, k, d, f, e_cnt, cap) -> int:
    return int(load_library().moe_workspace_bytes(which, dtype, T, k, d, f, e_cnt, cap))


def moe_route(logits, k, gate_mode, e_lo, e_cnt, topk_idx, topk_w, counts):
    import torch
    T, E = logits.shape
    _need(logits, torch.float32, name="logits")
    _need(topk_idx, torch.int32, (T, k), "topk_idx")
    _need(topk_w, torch.float32, (T, k), "topk_w")
    _need(counts, torch.int32, (e_cnt,), "counts")
    _check(load_library().moe_route(_ptr(logits), T, E, k, gate_mode, e_lo, e_cnt, _ptr(topk_idx), _ptr(topk_w),
                                    _ptr(counts), _stream()), "moe_route")


def moe_dispatch(x, k, topk_idx, row_scale, e_lo, e_cnt, offsets, perm, inv, reuse_plan, xp, ws):
    import torch
    T, d = x.shape
    cap = xp.shape[0]
    _need(x, name="x"); _need(xp, x.dtype, (cap, d), "xp")
    _need(topk_idx, torch.int32, (T, k), "topk_idx")
    _need(row_scale, torch.float32, (T, k), "row_scale")
    _need(offsets, torch.int32, (e_cnt + 1,), "offsets")
    _need(perm, torch.int32, (cap,), "perm")
    _need(inv, torch.int32, (T, k), "inv")
    _need(ws, name="ws")
    _check(load_library().moe_dispatch(_ptr(x), _dtype_code(x), T, d, k, _ptr(topk_idx), _ptr(row_scale), e_lo, e_cnt,
                                       _ptr(offsets), _ptr(perm), _ptr(inv), int(reuse_plan), _ptr(xp), cap,
                                       _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream()),
           "moe_dispatch")


def moe_dispatch_static(x, k, topk_idx, row_scale, e_lo, e_cnt, offsets, perm, inv, xp, status=None):
    """moe_dispatch (plan + row move) on the library's built-in plan scratch: no workspace argument."""
    import torch
    T, d = x.shape
    cap = xp.shape[0]
    _need(x, name="x"); _need(xp, x.dtype, (cap, d), "xp")
    _need(topk_idx, torch.int32, (T, k), "topk_idx")
    _need(row_scale, torch.float32, (T, k), "row_scale")
    _need(offsets, torch.int32, (e_cnt + 1,), "offsets")
    _need(perm, torch.int32, (cap,), "perm")
    _need(inv, torch.int32, (T, k), "inv")
    _need(status, torch.int32, name="status")
    lib = load_library()
    _check(lib.moe_dispatch_static(_ptr(x), _dtype_code(x), T, d, k, _ptr(topk_idx), _ptr(row_scale), e_lo, e_cnt,
                                   _ptr(offsets), _ptr(perm), _ptr(inv), _ptr(xp), cap, _ptr(status), _stream()),
           "moe_dispatch_static")


def moe_expert_fwd(xp, offsets, w1, w3, w2, h1, h3, o, ws, a=None):
    import torch
    cap, d = xp.shape
    e_cnt, _, f = w1.shape
    _need(xp, name="xp"); _need(o, xp.dtype, (cap, d), "o")
    _need(w1, xp.dtype, (e_cnt, d, f), "w1"); _need(w3, xp.dtype, (e_cnt, d, f), "w3")
    _need(w2, xp.dtype, (e_cnt, f, d), "w2")
    _need(h1, xp.dtype, (cap, f), "h1"); _need(h3, xp.dtype, (cap, f), "h3"); _need(a, xp.dtype, (cap, f), "a")
    _need(offsets, torch.int32, (e_cnt + 1,), "offsets"); _need(ws, name="ws")
    _check(load_library().moe_expert_fwd(_ptr(xp), _dtype_code(xp), cap, d, f, e_cnt, _ptr(offsets), _ptr(w1), _ptr(w3),
                                         _ptr(w2), _ptr(h1), _ptr(h3), _ptr(a), _ptr(o), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream()), "moe_expert_fwd")


def moe_expert_bwd(xp, h1, h3, d_o, offsets, w1, w3, w2, dxp, dw1, dw3, dw2, accumulate, ws, a=None):
    import torch
    cap, d = xp.shape
    e_cnt, _, f = w1.shape
    dt = xp.dtype
    _need(xp, name="xp"); _need(h1, dt, (cap, f), "h1"); _need(h3, dt, (cap, f), "h3"); _need(a, dt, (cap, f), "a")
    _need(d_o, dt, (cap, d), "d_o"); _need(dxp, dt, (cap, d), "dxp")
    _need(w1, dt, (e_cnt, d, f), "w1"); _need(w3, dt, (e_cnt, d, f), "w3"); _need(w2, dt, (e_cnt, f, d), "w2")
    _need(dw1, dt, (e_cnt, d, f), "dw1"); _need(dw3, dt, (e_cnt, d, f), "dw3"); _need(dw2, dt, (e_cnt, f, d), "dw2")
    _need(offsets, torch.int32, (e_cnt + 1,), "offsets"); _need(ws, name="ws")
    _check(load_library().moe_expert_bwd(_ptr(xp), _ptr(h1), _ptr(h3), _ptr(a), _ptr(d_o), _dtype_code(xp), cap, d, f, e_cnt,
                                         _ptr(offsets), _ptr(w1), _ptr(w3), _ptr(w2), _ptr(dxp), _ptr(dw1), _ptr(dw3),
                                         _ptr(dw2), int(accumulate), _ptr(ws), ws.numel() * ws.element_size(),
                                         _stream()), "moe_expert_bwd")


def moe_combine(o, inv, topk_w, y):
    import torch
    T, k = inv.shape
    d = o.shape[1]
    _need(o, name="o"); _need(y, o.dtype, (T, d), "y")
    _need(inv, torch.int32, name="inv"); _need(topk_w, torch.float32, (T, k), "topk_w")
    _check(load_library().moe_combine(_ptr(o), _dtype_code(o), T, d, k, _ptr(inv), _ptr(topk_w), _ptr(y), _stream()),
           "moe_combine")


def moe_router_fwd(x, wr, logits, ws):
    import torch
    T, d = x.shape
    E = wr.shape[1]
    _need(x, name="x"); _need(wr, x.dtype, (d, E), "wr"); _need(logits, torch.float32, (T, E), "logits")
    _need(ws, name="ws")
    _check(load_library().moe_router_fwd(_ptr(x), _ptr(wr), _dtype_code(x), T, d, E, _ptr(logits), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream()), "moe_router_fwd")


def moe_combine_bwd(dy, o, inv, topk_w, d_o, dgate):
    import torch
    T, k = inv.shape
    d = dy.shape[1]
    _need(dy, name="dy"); _need(o, dy.dtype, name="o"); _need(d_o, dy.dtype, tuple(o.shape), "d_o")
    _need(inv, torch.int32, name="inv"); _need(topk_w, torch.float32, (T, k), "topk_w")
    _need(dgate, torch.float32, (T, k), "dgate")
    if o.shape[1] != d or dy.shape[0] != T:
        raise MoeError("dy must be [T,d] and o [rows,d]")
    _check(load_library().moe_combine_bwd(_ptr(dy), _ptr(o), _dtype_code(dy), T, d, k, _ptr(inv), _ptr(topk_w),
                                          _ptr(d_o), _ptr(dgate), _stream()), "moe_combine_bwd")


def moe_gate_bwd(logits, topk_idx, dgate, gate_mode, dlogits):
    import torch
    T, E = logits.shape
    k = topk_idx.shape[1]
    _need(logits, torch.float32, name="logits"); _need(topk_idx, torch.int32, (T, k), "topk_idx")
    _need(dgate, torch.float32, (T, k), "dgate"); _need(dlogits, torch.float32, (T, E), "dlogits")
    _check(load_library().moe_gate_bwd(_ptr(logits), _ptr(topk_idx), _ptr(dgate), T, E, k, gate_mode, _ptr(dlogits),
                                       _stream()), "moe_gate_bwd")


def moe_router_bwd(x, wr, dlogits, dwr, dwr_accumulate, dx, dx_accumulate, ws):
    import torch
    T, d = x.shape
    E = wr.shape[1]
    _need(x, name="x"); _need(wr, x.dtype, (d, E), "wr"); _need(dlogits, torch.float32, (T, E), "dlogits")
    _need(dwr, x.dtype, (d, E), "dwr"); _need(dx, x.dtype, (T, d), "dx"); _need(ws, name="ws")
    _check(load_library().moe_router_bwd(_ptr(x), _ptr(wr), _ptr(dlogits), _dtype_code(x), T, d, E, _ptr(dwr),
                                         int(dwr_accumulate), _ptr(dx), int(dx_accumulate), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream()), "moe_router_bwd")


KERNEL_IDS = dict(route=0, plan=1, dispatch=2, combine=3, up=4, down=5, da=6, dx=7, wg=8, wgd=9, router_fwd=10,
                  combine_bwd=11, gate_bwd=12, router_dw=13, router_dx=14, wgrad_reduce=15, da_wg=16, dx_wgd=17)


def moe_profile_enable(on: bool):
    lib = load_library()
    lib.moe_profile_enable.restype = ctypes.c_int
    lib.moe_profile_enable.argtypes = [ctypes.c_int]
    _check(lib.moe_profile_enable(int(on)), "moe_profile_enable")


def moe_profile_read(kernel: str):
    """(total milliseconds, launches) recorded for one kernel family since profiling was enabled."""
    lib = load_library()
    lib.moe_profile_read.restype = ctypes.c_int
    lib.moe_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
    ms, n = ctypes.c_double(0), ctypes.c_int(0)
    _check(lib.moe_profile_read(KERNEL_IDS[kernel], ctypes.byref(ms), ctypes.byref(n)), "moe_profile_read")
    return ms.value, n.value


def moe_profile_stats(kernel: str):
    """(shortest, median) launch in milliseconds of one kernel family since profiling was enabled."""
    lib = load_library()
    lib.moe_profile_stats.restype = ctypes.c_int
    lib.moe_profile_stats.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lo, med = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib.moe_profile_stats(KERNEL_IDS[kernel], ctypes.byref(lo), ctypes.byref(med)), "moe_profile_stats")
    return lo.value, med.value


def moe_probe_mfma_bf16(sink, iters: int, random_operands: bool) -> float:
    """Enqueue the MFMA-only ceiling kernel; returns the FLOP count of the launch."""
    lib = load_library()
    lib.moe_probe_mfma_bf16.restype = ctypes.c_int
    lib.moe_probe_mfma_bf16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    flop = ctypes.c_double(0)
    _check(lib.moe_probe_mfma_bf16(_ptr(sink), sink.numel() * sink.element_size(), int(iters), int(random_operands),
                                   ctypes.byref(flop), _stream()), "moe_probe_mfma_bf16")
    return flop.value


def moe_probe_copy(src, dst):
    lib = load_library()
    lib.moe_probe_copy.restype = ctypes.c_int
    lib.moe_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    _check(lib.moe_probe_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()), "moe_probe_copy")


def moe_probe_mfma_fed_bf16(sink, iters: int, feed: int) -> float:
    """Enqueue the MFMA loop whose operands are re-read from LDS (feed 1: 16-byte reads, 2: transposing
    reads); returns the FLOP count of the launch."""
    lib = load_library()
    lib.moe_probe_mfma_fed_bf16.restype = ctypes.c_int
    lib.moe_probe_mfma_fed_bf16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                            ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    flop = ctypes.c_double(0)
    _check(lib.moe_probe_mfma_fed_bf16(_ptr(sink), sink.numel() * sink.element_size(), int(iters), int(feed),
                                       ctypes.byref(flop), _stream()), "moe_probe_mfma_fed_bf16")
    return flop.value


def moe_probe_stream(src, dst, writes: int, sink=None):
    """Streaming ceiling kernels over src's bytes: writes = -1 read only, 0 fill dst, n >= 1 one read and n writes."""
    lib = load_library()
    lib.moe_probe_stream.restype = ctypes.c_int
    lib.moe_probe_stream.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p,
                                     ctypes.c_void_p]
    nbytes = src.numel() * src.element_size()
    if writes >= 1 and dst.numel() * dst.element_size() < writes * nbytes:
        raise MoeError("dst must hold `writes` copies of src")
    _check(lib.moe_probe_stream(_ptr(src), _ptr(dst), nbytes, int(writes), _ptr(sink), _stream()), "moe_probe_stream")
