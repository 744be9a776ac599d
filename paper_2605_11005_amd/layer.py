"""Buffer plumbing for one MoE expert layer step: device allocations (torch is used for
memory and streams only) and the order in which the C entry points are enqueued.

forward : moe_route -> moe_dispatch (plan + row move) -> moe_expert_fwd -> moe_combine
backward: moe_dispatch(dy, row_scale=gate, reuse_plan) -> moe_expert_bwd -> moe_combine(dxp, no gate)
With the trainable gate (run_forward_router / run_backward_router):
forward : moe_router_fwd -> the forward above
backward: moe_combine_bwd (d_o and dgate in one pass) -> moe_expert_bwd -> moe_combine(dxp)
          -> moe_gate_bwd -> moe_router_bwd (dWr, and the router term added into dx)
Nothing synchronises with the host between the calls.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def torch_dtype(wl):
    return torch.bfloat16 if wl.dtype == "bf16" else torch.float32


def to_device(a: np.ndarray, dtype, bits: bool = False):
    """Host array -> device tensor.  bits=True: `a` is uint16 bf16 bit patterns."""
    if bits:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.cuda().to(dtype) if dtype != t.dtype else t.cuda()


def upload(wl, x, logits, dy, w1, w3, w2, bits: bool = False):
    dt = torch_dtype(wl)
    return dict(x=to_device(x, dt), logits=to_device(logits, torch.float32), dy=to_device(dy, dt),
                w1=to_device(w1, dt, bits), w3=to_device(w3, dt, bits), w2=to_device(w2, dt, bits))


class MoeLayerBuffers:
    """All outputs, saved activations and scratch of one layer step, allocated once."""

    def __init__(self, wl, cap: int, device="cuda", grads: bool = True, router: bool = False):
        dt = torch_dtype(wl)
        code = B.MOE_BF16 if wl.dtype == "bf16" else B.MOE_F32
        T, d, k, f, ec = wl.T, wl.d, wl.k, wl.f, wl.e_cnt
        self.cap = cap
        i32 = dict(dtype=torch.int32, device=device)
        self.topk_idx = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=device)
        self.counts = torch.empty((ec,), **i32)
        self.offsets = torch.empty((ec + 1,), **i32)
        self.perm = torch.empty((cap,), **i32)
        self.inv = torch.empty((T, k), **i32)
        self.xp = torch.empty((cap, d), dtype=dt, device=device)
        self.h1 = torch.empty((cap, f), dtype=dt, device=device)
        self.h3 = torch.empty((cap, f), dtype=dt, device=device)
        self.o = torch.empty((cap, d), dtype=dt, device=device)
        self.y = torch.empty((T, d), dtype=dt, device=device)
        nb = lambda which: B.moe_workspace_bytes(which, code, T, k, d, f, ec, cap)
        self.ws_dispatch = torch.empty(nb(B.WS_DISPATCH), dtype=torch.uint8, device=device)
        self.ws_fwd = torch.empty(nb(B.WS_EXPERT_FWD), dtype=torch.uint8, device=device)
        self.a = None
        if grads:
            self.a = torch.empty((cap, f), dtype=dt, device=device)      # kept by the forward for the backward
            self.d_o = torch.empty((cap, d), dtype=dt, device=device)
            self.dxp = torch.empty((cap, d), dtype=dt, device=device)
            self.dx = torch.empty((T, d), dtype=dt, device=device)
            self.dw1 = torch.empty((ec, d, f), dtype=dt, device=device)
            self.dw3 = torch.empty((ec, d, f), dtype=dt, device=device)
            self.dw2 = torch.empty((ec, f, d), dtype=dt, device=device)
            self.ws_bwd = torch.empty(nb(B.WS_EXPERT_BWD), dtype=torch.uint8, device=device)

        if router:
            E = wl.E
            self.logits = torch.empty((T, E), dtype=torch.float32, device=device)
            self.dgate = torch.empty((T, k), dtype=torch.float32, device=device)
            self.dlogits = torch.empty((T, E), dtype=torch.float32, device=device)
            self.dwr = torch.empty((d, E), dtype=dt, device=device)
            self.ws_router = torch.empty(B.moe_workspace_bytes(B.WS_ROUTER, code, T, k, d, f, E, cap), dtype=torch.uint8,
                                         device=device)

    def status(self) -> int:
        """Plan status word (1 = cap was too small).  Synchronises."""
        return int(self.ws_dispatch[:4].view(torch.int32).item())


def run_forward(wl, dev, buf: MoeLayerBuffers):
    B.moe_route(dev["logits"], wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt, buf.topk_idx, buf.topk_w, buf.counts)
    B.moe_dispatch(dev["x"], wl.k, buf.topk_idx, None, wl.e_lo, wl.e_cnt, buf.offsets, buf.perm, buf.inv, False,
                   buf.xp, buf.ws_dispatch)
    B.moe_expert_fwd(buf.xp, buf.offsets, dev["w1"], dev["w3"], dev["w2"], buf.h1, buf.h3, buf.o, buf.ws_fwd, a=buf.a)
    B.moe_combine(buf.o, buf.inv, buf.topk_w, buf.y)


def run_backward(wl, dev, buf: MoeLayerBuffers, accumulate: bool = False):
    B.moe_dispatch(dev["dy"], wl.k, None, buf.topk_w, wl.e_lo, wl.e_cnt, buf.offsets, buf.perm, buf.inv, True,
                   buf.d_o, None)
    B.moe_expert_bwd(buf.xp, buf.h1, buf.h3, buf.d_o, buf.offsets, dev["w1"], dev["w3"], dev["w2"], buf.dxp,
                     buf.dw1, buf.dw3, buf.dw2, accumulate, buf.ws_bwd, a=buf.a)
    B.moe_combine(buf.dxp, buf.inv, None, buf.dx)


def run_forward_router(wl, dev, buf: MoeLayerBuffers):
    """Forward with the router GEMM inside the library: dev needs "x" and "wr"."""
    B.moe_router_fwd(dev["x"], dev["wr"], buf.logits, buf.ws_router)
    B.moe_route(buf.logits, wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt, buf.topk_idx, buf.topk_w, buf.counts)
    B.moe_dispatch(dev["x"], wl.k, buf.topk_idx, None, wl.e_lo, wl.e_cnt, buf.offsets, buf.perm, buf.inv, False,
                   buf.xp, buf.ws_dispatch)
    B.moe_expert_fwd(buf.xp, buf.offsets, dev["w1"], dev["w3"], dev["w2"], buf.h1, buf.h3, buf.o, buf.ws_fwd, a=buf.a)
    B.moe_combine(buf.o, buf.inv, buf.topk_w, buf.y)


def run_backward_router(wl, dev, buf: MoeLayerBuffers, accumulate: bool = False):
    """Backward including the gate: dx = expert-path term + router term; dwr = gradient of Wr."""
    B.moe_combine_bwd(dev["dy"], buf.o, buf.inv, buf.topk_w, buf.d_o, buf.dgate)
    B.moe_expert_bwd(buf.xp, buf.h1, buf.h3, buf.d_o, buf.offsets, dev["w1"], dev["w3"], dev["w2"], buf.dxp,
                     buf.dw1, buf.dw3, buf.dw2, accumulate, buf.ws_bwd, a=buf.a)
    B.moe_combine(buf.dxp, buf.inv, None, buf.dx)
    B.moe_gate_bwd(buf.logits, buf.topk_idx, buf.dgate, wl.gate_mode, buf.dlogits)
    B.moe_router_bwd(dev["x"], dev["wr"], buf.dlogits, buf.dwr, accumulate, buf.dx, True, buf.ws_router)
