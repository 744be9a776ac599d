"""Token-chunked, two-stream schedule of the expert layer on one GPU.

The paper's operator-level overlap (section on the unlocked operation-level overlapping space:
the GroupGEMM in the FFN admits natural chunking, so that dispatch/combine of one chunk can run
beside the GEMMs of another) applied to the one part that exists on a single GPU: the local row
movers against the grouped GEMMs.  The tokens are cut into contiguous chunks; chunk c's
route/plan/dispatch/combine kernels are enqueued on a "mover" stream, its grouped GEMMs on a
"gemm" stream, with events carrying the dependencies, so the movers of chunk c+1 may overlap the
GEMMs of chunk c.  Weight gradients accumulate over the chunks in chunk order on the gemm stream
(accumulate = 1 from the second chunk on), so results stay reproducible.

Every arithmetic step still runs in the library's kernels; this module only orders the calls.
Outputs per token (y, dx) are bit-identical to the unchunked schedule: a row's GEMM results do not
depend on which other rows share its tile.  Weight gradients differ by one bf16 rounding per chunk.
"""
from __future__ import annotations

from dataclasses import replace

import torch

from . import binding as B
from .layer import MoeLayerBuffers


class ChunkedLayer:
    """Buffers and streams for `n_chunks` token chunks of workload `wl` (T divisible by n_chunks).
    `caps[c]` = rows available to chunk c (its routed row count, or T_c * min(k, e_cnt))."""

    def __init__(self, wl, n_chunks: int, caps=None):
        if wl.T % n_chunks:
            raise ValueError("T must be divisible by the number of chunks")
        self.wl, self.n = wl, n_chunks
        self.Tc = wl.T // n_chunks
        self.wlc = replace(wl, T=self.Tc)
        caps = caps or [self.Tc * min(wl.k, wl.e_cnt)] * n_chunks
        self.bufs = [MoeLayerBuffers(self.wlc, cap=max(int(c), 1)) for c in caps]
        # weight gradients are shared by all chunks
        for b in self.bufs[1:]:
            b.dw1, b.dw3, b.dw2 = self.bufs[0].dw1, self.bufs[0].dw3, self.bufs[0].dw2
        self.mover = torch.cuda.Stream()
        self.gemm = torch.cuda.Stream()

    def _ev(self, stream):
        e = torch.cuda.Event()
        e.record(stream)
        return e

    def forward(self, dev):
        wl, Tc = self.wlc, self.Tc
        cur = torch.cuda.current_stream()
        start = self._ev(cur)
        self.mover.wait_event(start); self.gemm.wait_event(start)
        done = []
        for c, buf in enumerate(self.bufs):
            x = dev["x"][c * Tc:(c + 1) * Tc]
            lg = dev["logits"][c * Tc:(c + 1) * Tc]
            with torch.cuda.stream(self.mover):
                B.moe_route(lg, wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt, buf.topk_idx, buf.topk_w, buf.counts)
                B.moe_dispatch(x, wl.k, buf.topk_idx, None, wl.e_lo, wl.e_cnt, buf.offsets, buf.perm, buf.inv, False,
                               buf.xp, buf.ws_dispatch)
                moved = self._ev(self.mover)
            with torch.cuda.stream(self.gemm):
                self.gemm.wait_event(moved)
                B.moe_expert_fwd(buf.xp, buf.offsets, dev["w1"], dev["w3"], dev["w2"], buf.h1, buf.h3, buf.o, buf.ws_fwd)
                computed = self._ev(self.gemm)
            with torch.cuda.stream(self.mover):
                self.mover.wait_event(computed)
                B.moe_combine(buf.o, buf.inv, buf.topk_w, buf.y)
                done.append(self._ev(self.mover))
        for e in done:
            cur.wait_event(e)

    def backward(self, dev):
        wl, Tc = self.wlc, self.Tc
        cur = torch.cuda.current_stream()
        start = self._ev(cur)
        self.mover.wait_event(start); self.gemm.wait_event(start)
        done = []
        for c, buf in enumerate(self.bufs):
            dy = dev["dy"][c * Tc:(c + 1) * Tc]
            with torch.cuda.stream(self.mover):
                B.moe_dispatch(dy, wl.k, None, buf.topk_w, wl.e_lo, wl.e_cnt, buf.offsets, buf.perm, buf.inv, True,
                               buf.d_o, None)
                moved = self._ev(self.mover)
            with torch.cuda.stream(self.gemm):
                self.gemm.wait_event(moved)
                B.moe_expert_bwd(buf.xp, buf.h1, buf.h3, buf.d_o, buf.offsets, dev["w1"], dev["w3"], dev["w2"], buf.dxp,
                                 buf.dw1, buf.dw3, buf.dw2, c > 0, buf.ws_bwd)
                computed = self._ev(self.gemm)
            with torch.cuda.stream(self.mover):
                self.mover.wait_event(computed)
                B.moe_combine(buf.dxp, buf.inv, None, buf.dx)
                done.append(self._ev(self.mover))
        for e in done:
            cur.wait_event(e)

    def y(self):
        return torch.cat([b.y for b in self.bufs])

    def dx(self):
        return torch.cat([b.dx for b in self.bufs])
