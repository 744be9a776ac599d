"""GPU parity of the trainable gate (router GEMM, fused backward of combine, gradient through
the gate weights, router backward) against the CPU oracle, through the C ABI.

The router's logits are compared with the oracle's first; from there on both sides continue from
the GPU's logits (uploaded bit for bit), so that a near-tie decided differently by two summation
orders cannot turn into a different selection.  Each backward step is compared twice: against the
oracle's own chain (the end-to-end tolerance of the dtype) and, for the element-wise gate step,
against the oracle fed with the GPU's inputs (fp32 tolerance)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2605_11005_amd import binding as B
from paper_2605_11005_amd import workloads as W
from paper_2605_11005_amd.layer import MoeLayerBuffers, run_backward_router, run_forward_router, to_device, torch_dtype
from tests.gpu_util import TOL, host, rel_err

pytestmark = pytest.mark.gpu

CASES = [
    W.TINY,                                                                         # fp32, E = 8: plain path
    W.TINY.scaled(name="tiny-fp32-softmax", gate_mode=W.GATE_SOFTMAX, T=300, E=12, e_lo=3, e_cnt=5, k=3, d=72, f=100),
    W.TINY.scaled(name="tiny-fp32-sigmoid", gate_mode=W.GATE_SIGMOID_RENORM, T=130, E=70, e_lo=0, e_cnt=70, k=6, d=40, f=36),
    W.MIXTRAL.scaled(name="mixtral-small-router", T=2048, d=256, f=384),           # bf16, E = 8: plain path on bf16
    W.QWEN.scaled(name="qwen-small-router", T=2048, d=256, f=192),                 # bf16, E = 128: matrix cores
    W.DSV3.scaled(name="dsv3-small-router", T=4096, d=512, f=256),                 # E = 256, sigmoid gate
    W.DSV3.scaled(name="ragged-router", T=1500, d=320, f=448, E=96, e_lo=8, e_cnt=8, k=6),      # tails in every dimension
    W.QWEN.scaled(name="softmax-router", gate_mode=W.GATE_SOFTMAX, T=777, d=128, f=64, E=160, e_lo=32, e_cnt=64, k=4),
    # few logit tiles and a long contraction: the router GEMM cuts d into five ranges of 5, 5, 5, 5 and 3 pairs of
    # k-tiles and adds their fp32 tiles up; the token count leaves a ragged last row tile
    W.QWEN.scaled(name="cut-contraction-router", T=1000, d=1472, f=64, E=128, e_lo=16, e_cnt=16, k=4),
]


def _random_router_cases(n, seed):
    """Seeded draws for the matrix-core router path (E and d multiples of 64): token counts with ragged
    last tiles, contractions from one pair of k-tiles to 24 (cut into up to five ranges), any slice."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        E = 64 * int(rng.integers(1, 5))
        e_cnt = int(rng.integers(1, 33))
        e_lo = int(rng.integers(0, E - e_cnt + 1))
        out.append(W.DSV3.scaled(name=f"random-router-{seed}-{i}", T=int(rng.integers(1, 2500)), d=64 * int(rng.integers(1, 25)),
                                 f=64 * int(rng.integers(1, 3)), E=E, e_lo=e_lo, e_cnt=e_cnt, k=int(rng.integers(1, 9)),
                                 gate_mode=int(rng.integers(0, 3)), zipf_s=float(rng.choice([0.0, 1.0]))))
    return out


@pytest.mark.parametrize("wl", CASES + _random_router_cases(6, 20260512), ids=lambda w: w.name)
def test_trainable_gate_forward_backward(wl):
    print(f"case {wl.name} T={wl.T} d={wl.d} f={wl.f} E={wl.E} slice=[{wl.e_lo},{wl.e_lo + wl.e_cnt}) k={wl.k} "
          f"gate={wl.gate_mode} {wl.dtype}", flush=True)
    tol = TOL[wl.dtype]
    x = W.tokens(wl); wr = W.router_weights(wl); dy = W.out_grad(wl)
    w1, w3, w2 = W.all_expert_weights(wl)
    dt = torch_dtype(wl)
    dev = dict(x=to_device(x, dt), wr=to_device(wr, dt), dy=to_device(dy, dt), w1=to_device(w1, dt),
               w3=to_device(w3, dt), w2=to_device(w2, dt))
    buf = MoeLayerBuffers(wl, cap=wl.T * min(wl.k, wl.e_cnt), router=True)
    for name in ("logits", "dgate", "dlogits", "dwr", "d_o", "dx"):
        getattr(buf, name).fill_(7.0)
    run_forward_router(wl, dev, buf)
    run_backward_router(wl, dev, buf)
    torch.cuda.synchronize()
    errs = {}
    # router GEMM: both sides accumulate the same products, the oracle in float64
    logits_ref = O.router_logits(x, wr)
    logits = host(buf.logits).astype(np.float32)
    errs["logits"] = rel_err(logits, logits_ref)
    assert errs["logits"] < 1e-5, errs
    # from here on: the GPU's logits on both sides
    fw = O.layer_fwd(x, logits, wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt, w1, w3, w2)
    bw = O.layer_bwd(fw, dy, wl.k, w1, w3, w2)
    R = int(fw["offsets"][-1])
    assert (host(buf.topk_idx) == fw["topk_idx"]).all()
    assert (host(buf.inv) == fw["inv"]).all()
    errs["y"] = rel_err(host(buf.y), fw["y"])
    errs["d_o"] = rel_err(host(buf.d_o[:R]), bw["d_o"])
    dg = O.gate_grad(dy, fw["o"], fw["inv"])
    dg_gpu = host(buf.dgate)
    errs["dgate"] = rel_err(dg_gpu, dg)
    assert not dg_gpu[fw["inv"] < 0].any(), "dgate of a slot without a local expert must be zero"
    dl = O.gate_bwd(logits, fw["topk_idx"], dg, wl.gate_mode)
    errs["dlogits"] = rel_err(host(buf.dlogits), dl)
    # the gate step alone, fed with the GPU's own dgate: fp32 arithmetic on both sides
    dl_iso = O.gate_bwd(logits, fw["topk_idx"], dg_gpu, wl.gate_mode)
    errs["dlogits_iso"] = rel_err(host(buf.dlogits), dl_iso)
    assert errs["dlogits_iso"] < 1e-5, errs
    dwr, dx_r = O.router_bwd(x, wr, dl)
    errs["dwr"] = rel_err(host(buf.dwr), dwr)
    errs["dx_total"] = rel_err(host(buf.dx), bw["dx"] + dx_r)
    # the router GEMMs alone, fed with the GPU's dlogits
    dwr_iso, dx_r_iso = O.router_bwd(x, wr, host(buf.dlogits))
    errs["dwr_iso"] = rel_err(host(buf.dwr), dwr_iso)
    print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v < tol}
    assert not bad, bad
    assert np.abs(dx_r).max() > 0 and np.abs(dwr).max() > 0


def test_router_bwd_overwrite_accumulate_and_skips():
    wl = W.QWEN.scaled(name="router-acc", T=600, d=128, f=64, E=64, e_lo=0, e_cnt=64, k=4)
    rng = np.random.default_rng(5)
    x = W.tokens(wl); wr = W.router_weights(wl)
    dl = rng.standard_normal((wl.T, wl.E)).astype(np.float32)
    dt = torch.bfloat16
    dx0 = rng.standard_normal((wl.T, wl.d)).astype(np.float32)
    xd, wrd, dld = to_device(x, dt), to_device(wr, dt), to_device(dl, torch.float32)
    ws = torch.empty(B.moe_workspace_bytes(B.WS_ROUTER, B.MOE_BF16, wl.T, wl.k, wl.d, wl.f, wl.E, 0), dtype=torch.uint8, device="cuda")
    dwr_ref, dxr_ref = O.router_bwd(x, wr, dl)
    dwr = torch.full((wl.d, wl.E), 3.0, dtype=dt, device="cuda")
    dx = to_device(dx0, dt)
    dx0r = host(dx)
    B.moe_router_bwd(xd, wrd, dld, dwr, False, dx, True, ws)
    torch.cuda.synchronize()
    assert rel_err(host(dwr), dwr_ref) < 2e-2
    assert rel_err(host(dx), dx0r + dxr_ref) < 2e-2
    first = host(dwr)
    B.moe_router_bwd(xd, wrd, dld, dwr, True, dx, False, ws)
    torch.cuda.synchronize()
    assert rel_err(host(dwr), 2 * first) < 1e-2
    assert rel_err(host(dx), dxr_ref) < 2e-2
    keep = dwr.clone()
    B.moe_router_bwd(xd, wrd, dld, None, False, dx, False, ws)       # dWr skipped
    torch.cuda.synchronize()
    assert torch.equal(keep, dwr)


def test_combine_bwd_matches_scaled_dispatch_bit_for_bit():
    """d_o from the fused pass equals the scaled moe_dispatch exactly (same products, one rounding)."""
    wl = W.DSV3.scaled(name="cb-vs-dispatch", T=3000, d=1024, f=64)
    from tests.gpu_util import gpu_layer, make_inputs
    inp = make_inputs(wl)
    dev, buf = gpu_layer(wl, inp)
    d_o2 = torch.full_like(buf.d_o, 5.0)
    dgate = torch.empty((wl.T, wl.k), dtype=torch.float32, device="cuda")
    B.moe_combine_bwd(dev["dy"], buf.o, buf.inv, buf.topk_w, d_o2, dgate)
    torch.cuda.synchronize()
    R = int(buf.offsets[-1])
    assert torch.equal(d_o2[:R], buf.d_o[:R])
    dgate2 = torch.empty_like(dgate)
    B.moe_combine_bwd(dev["dy"], buf.o, buf.inv, buf.topk_w, d_o2, dgate2)
    torch.cuda.synchronize()
    assert torch.equal(dgate, dgate2), "the reduction order is fixed: bit-identical run to run"


def test_trainable_gate_full_size_sampled():
    """The gate kernels at the DeepSeek-V3-like share, in the launch configuration bench.py times.
    Compared on what the oracle can compute one by one: logits of sampled tokens, dgate of sampled
    tokens (from the GPU's own o rows), dlogits in full (element-wise step), sampled columns of dWr
    over all tokens, and the router term of dx on sampled tokens."""
    wl = W.DSV3
    print(f"full-size gate case {wl.name}: T={wl.T} d={wl.d} E={wl.E} k={wl.k}", flush=True)
    rng = np.random.default_rng(wl.seed)
    x = W.tokens(wl); wr = W.router_weights(wl); dy = W.out_grad(wl)
    dt = torch.bfloat16
    xd, wrd, dyd = to_device(x, dt), to_device(wr, dt), to_device(dy, dt)
    T, d, E, k = wl.T, wl.d, wl.E, wl.k
    ws = torch.empty(B.moe_workspace_bytes(B.WS_ROUTER, B.MOE_BF16, T, k, d, wl.f, E, 0), dtype=torch.uint8, device="cuda")
    logits = torch.full((T, E), 7.0, dtype=torch.float32, device="cuda")
    B.moe_router_fwd(xd, wrd, logits, ws)
    ti = torch.empty((T, k), dtype=torch.int32, device="cuda"); tw = torch.empty((T, k), device="cuda")
    cnt = torch.empty((wl.e_cnt,), dtype=torch.int32, device="cuda")
    B.moe_route(logits, k, wl.gate_mode, wl.e_lo, wl.e_cnt, ti, tw, cnt)
    R = int(cnt.sum().item())
    off = torch.empty((wl.e_cnt + 1,), dtype=torch.int32, device="cuda")
    perm = torch.empty((R,), dtype=torch.int32, device="cuda"); inv = torch.empty_like(ti)
    wsd = torch.empty(B.moe_workspace_bytes(B.WS_DISPATCH, B.MOE_BF16, T, k, d, wl.f, wl.e_cnt, R), dtype=torch.uint8, device="cuda")
    xp = torch.empty((R, d), dtype=dt, device="cuda")
    B.moe_dispatch(xd, k, ti, None, wl.e_lo, wl.e_cnt, off, perm, inv, False, xp, wsd)
    o = torch.randn((R, d), device="cuda", dtype=dt)          # stands in for the expert outputs
    d_o = torch.empty_like(o); dgate = torch.full((T, k), 7.0, device="cuda")
    B.moe_combine_bwd(dyd, o, inv, tw, d_o, dgate)
    dlog = torch.full((T, E), 7.0, device="cuda")
    B.moe_gate_bwd(logits, ti, dgate, wl.gate_mode, dlog)
    dwr = torch.full((d, E), 7.0, dtype=dt, device="cuda")
    dx = torch.zeros((T, d), dtype=dt, device="cuda")
    B.moe_router_bwd(xd, wrd, dlog, dwr, False, dx, False, ws)
    torch.cuda.synchronize()
    # logits of sampled tokens
    rows = np.sort(rng.choice(T, size=512, replace=False))
    lg = host(logits)
    assert rel_err(lg[rows], O.router_logits(x[rows], wr)) < 1e-5
    # selection on the GPU's logits, in full
    ti_ref, tw_ref, cnt_ref = O.route(lg.astype(np.float32), k, wl.gate_mode, wl.e_lo, wl.e_cnt)
    assert (host(ti) == ti_ref).all() and (host(cnt) == cnt_ref).all()
    # dgate of sampled tokens from the GPU's o rows
    inv_h = host(inv)
    o_h = host(o)
    dg_ref = O.gate_grad(dy[rows], o_h, inv_h[rows])
    dg = host(dgate)
    assert rel_err(dg[rows], dg_ref) < 2e-2
    assert not dg[inv_h < 0].any()
    # gate backward, element-wise: in full from the GPU's dgate
    dl_ref = O.gate_bwd(lg.astype(np.float32), ti_ref, dg, wl.gate_mode)
    dl = host(dlog)
    assert rel_err(dl, dl_ref) < 1e-5
    # sampled columns of dWr over all tokens; router term of dx on sampled tokens
    # (the pinned oracle function on slices: column J of dWr depends only on column J of dlogits,
    # row t of the router term of dx only on row t of dlogits)
    J = np.sort(rng.choice(E, size=6, replace=False))
    dwr_ref, _ = O.router_bwd(x, wr[:, J], dl[:, J])
    assert rel_err(host(dwr)[:, J], dwr_ref) < 2e-2
    _, dx_ref = O.router_bwd(x[rows], wr, dl[rows])
    assert rel_err(host(dx)[rows], dx_ref) < 2e-2


def test_router_calls_with_more_tokens_than_one_grid_dimension_holds():
    """T > 65535 with a handful of experts (the plain kernels): every launch shape must fit the grid limits."""
    T, d, E = 70000, 64, 8
    rng = np.random.default_rng(5)
    x = rng.standard_normal((T, d)).astype(np.float32)
    wr = (rng.standard_normal((d, E)) * d ** -0.5).astype(np.float32)
    dl = rng.standard_normal((T, E)).astype(np.float32)
    xd, wrd, dld = torch.from_numpy(x).cuda(), torch.from_numpy(wr).cuda(), torch.from_numpy(dl).cuda()
    ws = torch.empty(B.moe_workspace_bytes(B.WS_ROUTER, B.MOE_F32, T, 2, d, 64, E, 0), dtype=torch.uint8, device="cuda")
    logits = torch.full((T, E), 7.0, device="cuda")
    B.moe_router_fwd(xd, wrd, logits, ws)
    dwr = torch.full((d, E), 7.0, device="cuda"); dx = torch.full((T, d), 7.0, device="cuda")
    B.moe_router_bwd(xd, wrd, dld, dwr, False, dx, False, ws)
    torch.cuda.synchronize()
    assert rel_err(host(logits), O.router_logits(x, wr)) < 1e-5
    dwr_ref, dx_ref = O.router_bwd(x, wr, dl)
    assert rel_err(host(dwr), dwr_ref) < 1e-5
    assert rel_err(host(dx), dx_ref) < 1e-5
