"""moe_dispatch_static -- the entry point for callers that cannot allocate -- against moe_dispatch.

Called through the C ABI binding twice in a row, the second time with a smaller input, so that what
the first call left in the library's built-in scratch must not leak into the second.  Every output
(offsets, perm, inv, the moved rows, the status word) must be bit-identical to moe_dispatch's, which
the other GPU tests hold to the oracle.  The allocator's counters must not move across the calls."""
import numpy as np
import pytest
import torch

from paper_2605_11005_amd import binding as B
from paper_2605_11005_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(wl, cap_delta=0, scaled=False):
    x = W.tokens(wl)
    logits = W.router_logits(wl, x)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    xd = torch.from_numpy(x).cuda().to(dt)
    T, k, d, ec = wl.T, wl.k, wl.d, wl.e_cnt
    ti = torch.empty((T, k), dtype=torch.int32, device="cuda")
    tw = torch.empty((T, k), dtype=torch.float32, device="cuda")
    cnt = torch.empty((ec,), dtype=torch.int32, device="cuda")
    B.moe_route(torch.from_numpy(logits).cuda(), k, wl.gate_mode, wl.e_lo, ec, ti, tw, cnt)
    cap = max(int(cnt.sum().item()) + cap_delta, 1)
    scale = tw if scaled else None
    code = B.MOE_BF16 if wl.dtype == "bf16" else B.MOE_F32

    def bufs():
        return (torch.full((ec + 1,), -7, dtype=torch.int32, device="cuda"),
                torch.full((cap,), -7, dtype=torch.int32, device="cuda"),
                torch.full((T, k), -7, dtype=torch.int32, device="cuda"),
                torch.full((cap, d), float("nan"), dtype=dt, device="cuda"))

    off0, perm0, inv0, xp0 = bufs()
    ws = torch.zeros(B.moe_workspace_bytes(B.WS_DISPATCH, code, T, k, d, wl.f, ec, cap), dtype=torch.uint8, device="cuda")
    B.moe_dispatch(xd, k, ti, scale, wl.e_lo, ec, off0, perm0, inv0, False, xp0, ws)
    off1, perm1, inv1, xp1 = bufs()
    status = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    B.moe_dispatch_static(xd, k, ti, scale, wl.e_lo, ec, off1, perm1, inv1, xp1, status)   # first use looks the scratch up
    for t in (off1, perm1, inv1):
        t.fill_(-7)
    xp1.fill_(float("nan")); status.fill_(-7)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    free_before = torch.cuda.mem_get_info()[0]
    B.moe_dispatch_static(xd, k, ti, scale, wl.e_lo, ec, off1, perm1, inv1, xp1, status)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before
    assert torch.cuda.mem_get_info()[0] == free_before, "the call must not take device memory"
    R = int(off0[-1].item())
    assert torch.equal(off0, off1), "offsets"
    assert torch.equal(perm0[:R], perm1[:R]) and (perm1[R:] == -7).all(), "perm"
    assert torch.equal(inv0, inv1), "inv"
    assert torch.equal(xp0[:R].view(torch.int16 if dt == torch.bfloat16 else torch.int32),
                       xp1[:R].view(torch.int16 if dt == torch.bfloat16 else torch.int32)), "moved rows"
    assert torch.isnan(xp1[R:]).all(), "rows past R are left untouched"
    assert int(status.item()) == int(ws[:4].view(torch.int32).item()), "status word"
    return R, int(status.item())


def test_two_calls_in_a_row_second_smaller():
    big = W.DSV3.scaled(name="static-big", T=8192, d=512)
    small = W.DSV3.scaled(name="static-small", T=1000, d=256, E=64, e_lo=8, e_cnt=8, k=6)
    R1, st1 = _both(big)
    R2, st2 = _both(small, scaled=True)
    assert R1 > R2 > 0 and st1 == 0 and st2 == 0
    # a capacity that is too small: both entry points drop the same rows and raise the status word
    R3, st3 = _both(small, cap_delta=-29)
    assert st3 == 1 and R3 == R2 - 29
    # fp32 rows and an empty batch
    _both(W.TINY)
    _both(W.TINY.scaled(name="static-empty", T=0))
