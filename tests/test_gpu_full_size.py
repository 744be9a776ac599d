"""GPU parity at the full headline shapes, in the launch configuration bench.py times.

Every output buffer is filled with NaN before the step and must be finite afterwards in all rows
below R (all elements for the weight gradients), so a tile that no workgroup wrote fails.
The integer artefacts and the row movers are compared with the oracle in full.

Expert GEMMs:
* the two shapes the performance target is quoted on (the DeepSeek-V3-like share and its skewed
  variant) are compared IN FULL: for every local expert the oracle computes the expert's forward
  and backward on all of its rows, and h1, h3, o, dxp, dW1, dW3, dW2 are compared whole;
* the other shapes are compared on samples the oracle can compute one by one: for h1/h3/o/dxp at
  least 1024 random rows per picked expert (the hottest, a mid-sized one and the smallest
  non-empty one; each row of those outputs depends only on its own input row); for dW1/dW3/dW2
  a set of hidden units j of the same experts -- column j of dW1/dW3 and row j of dW2 depend only
  on hidden unit j, so the oracle is called with the weights sliced to those units and all rows
  of the expert.
Experts without rows must get exactly zero gradients.  Beside the max-norm error the tolerance
is stated on, the relative l2 error is held to the same bound and the element-wise relative
error (absolute floor 1e-3 * max|ref|) is printed."""
import time

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2605_11005_amd import workloads as W
from paper_2605_11005_amd.layer import MoeLayerBuffers, run_backward, run_forward, to_device, torch_dtype
from tests.gpu_util import TOL, elementwise_err, host, rel_err, rms_err

pytestmark = pytest.mark.gpu

FULL = {W.DSV3.name, W.SKEW.name}        # compared whole, expert by expert
SAMPLE_ROWS = 1024
SAMPLE_UNITS = 8


class Worst:
    """Largest max-norm / l2 / element-wise figures seen per output name."""

    def __init__(self):
        self.mx, self.l2, self.ew, self.ew_frac = {}, {}, {}, {}

    def add(self, name, got, ref):
        self.mx[name] = max(self.mx.get(name, 0.0), rel_err(got, ref))
        self.l2[name] = max(self.l2.get(name, 0.0), rms_err(got, ref))
        m, fr = elementwise_err(got, ref)
        self.ew[name] = max(self.ew.get(name, 0.0), m)
        self.ew_frac[name] = max(self.ew_frac.get(name, 0.0), fr)

    def report(self):
        f = lambda d: {k: f"{v:.2e}" for k, v in d.items()}
        print("  max-norm error     ", f(self.mx), flush=True)
        print("  relative l2 error  ", f(self.l2), flush=True)
        print("  element-wise (floor 1e-3 max|ref|): largest", f(self.ew), "fraction above 2e-2", f(self.ew_frac), flush=True)


@pytest.mark.parametrize("wl", [W.MIXTRAL, W.QWEN, W.DSV3, W.SKEW] + W.MODEL_TABLE, ids=lambda w: w.name)
def test_full_size_layer(wl):
    t0 = time.time()
    print(f"full-size case {wl.name}: T={wl.T} d={wl.d} f={wl.f} E={wl.E} local={wl.e_cnt} k={wl.k}", flush=True)
    x = W.tokens(wl); logits = W.router_logits(wl, x); dy = W.out_grad(wl)
    w1b, w3b, w2b = W.all_expert_weights(wl, out_bits=True)
    dt = torch_dtype(wl)
    dev = dict(x=to_device(x, dt), logits=to_device(logits, torch.float32), dy=to_device(dy, dt),
               w1=to_device(w1b, dt, True), w3=to_device(w3b, dt, True), w2=to_device(w2b, dt, True))
    del w1b, w3b, w2b
    # oracle: routing, plan, both dispatches, at full size
    ti, tw, cnt = O.route(logits, wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt)
    off, perm, inv = O.plan(ti, wl.e_lo, wl.e_cnt)
    R = int(off[-1])
    print(f"  inputs+oracle plan {time.time() - t0:.1f}s; R={R}; rows/expert min {cnt.min()} max {cnt.max()}", flush=True)
    buf = MoeLayerBuffers(wl, cap=max(R, 1))          # the capacity bench.py uses
    nan = float("nan")
    for name in ("xp", "h1", "h3", "o", "y", "d_o", "dxp", "dx", "dw1", "dw3", "dw2"):
        getattr(buf, name).fill_(nan)
    run_forward(wl, dev, buf)
    run_backward(wl, dev, buf)
    torch.cuda.synchronize()
    assert buf.status() == 0
    tol = TOL[wl.dtype]
    # ---- nothing the step owns is left unwritten
    for name in ("xp", "h1", "h3", "o", "d_o", "dxp"):
        assert torch.isfinite(getattr(buf, name)[:R]).all().item(), f"{name}: unwritten or non-finite element"
    for name in ("y", "dx", "dw1", "dw3", "dw2"):
        assert torch.isfinite(getattr(buf, name)).all().item(), f"{name}: unwritten or non-finite element"
    # ---- bit-exact integer artefacts
    assert (host(buf.topk_idx) == ti).all()
    assert (host(buf.counts) == cnt).all()
    assert (host(buf.offsets) == off).all()
    assert (host(buf.perm)[:R] == perm).all()
    assert (host(buf.inv) == inv).all()
    assert np.abs(host(buf.topk_w) - tw).max() < 1e-5
    # ---- row movers in full: xp is an exact copy, d_o = gate * dy rounded once
    xp_gpu = buf.xp[:R]
    rows_tok = torch.from_numpy(perm.astype(np.int64) // wl.k).cuda()
    assert torch.equal(xp_gpu, dev["x"][rows_tok]), "dispatch must copy rows exactly"
    gate = torch.from_numpy(tw.reshape(-1)[perm].astype(np.float32)).cuda()
    d_o_ref = dev["dy"][rows_tok].float() * gate[:, None]
    err = (buf.d_o[:R].float() - d_o_ref).abs().max().item() / d_o_ref.abs().max().item()
    assert err < 1e-2, err
    del d_o_ref, rows_tok
    # combine checked against the oracle's definition applied to the GPU's own o / dxp (isolates the row mover)
    o_host = host(buf.o[:R])
    y_ref = O.combine(o_host, inv, tw)
    assert rel_err(host(buf.y), y_ref) < 1e-2
    del y_ref, o_host
    dx_ref = O.combine(host(buf.dxp[:R]), inv, None)
    assert rel_err(host(buf.dx), dx_ref) < 1e-2
    del dx_ref
    # ---- expert GEMMs
    for e in range(wl.e_cnt):
        if cnt[e] == 0:
            for g in (buf.dw1, buf.dw3, buf.dw2):
                assert not g[e].any().item(), f"empty expert {e} must have zero gradients"
    worst = Worst()
    rng = np.random.default_rng(wl.seed)
    nonempty = [e for e in range(wl.e_cnt) if cnt[e] > 0]
    if wl.name in FULL:
        rows_checked = 0
        for e in nonempty:
            lo, hi = int(off[e]), int(off[e + 1])
            w1, w3, w2 = W.expert_weights(wl, e)
            xe = x[perm[lo:hi] // wl.k]
            one = np.array([0, hi - lo], dtype=np.int32)
            h1, h3, _, o = O.expert_fwd(xe, one, [w1], [w3], [w2])
            d_oe = O.dispatch(dy, perm[lo:hi], wl.k, row_scale=tw)
            dxp, dw1, dw3, dw2 = O.expert_bwd(xe, h1, h3, d_oe, one, [w1], [w3], [w2])
            for name, got, ref in (("h1", buf.h1[lo:hi], h1), ("h3", buf.h3[lo:hi], h3), ("o", buf.o[lo:hi], o),
                                   ("dxp", buf.dxp[lo:hi], dxp), ("dw1", buf.dw1[e], dw1[0]), ("dw3", buf.dw3[e], dw3[0]),
                                   ("dw2", buf.dw2[e], dw2[0])):
                worst.add(name, host(got), ref)
            del h1, h3, o, d_oe, dxp, dw1, dw3, dw2, xe
            rows_checked += hi - lo
            print(f"  expert {e}: all {hi - lo} rows and all weight gradients compared ({time.time() - t0:.1f}s)", flush=True)
        assert rows_checked == R
    else:
        order = sorted(nonempty, key=lambda e: cnt[e])
        picks = sorted({order[-1], order[len(order) // 2], order[0]})
        for e in picks:
            lo, hi = int(off[e]), int(off[e + 1])
            n = hi - lo
            w1, w3, w2 = W.expert_weights(wl, e)
            # (a) sampled rows: h1, h3, o, dxp
            rs = np.sort(rng.choice(n, size=min(n, SAMPLE_ROWS), replace=False)) + lo
            xs = x[perm[rs] // wl.k].astype(np.float64)
            one = np.array([0, len(rs)], dtype=np.int32)
            h1, h3, a, o = O.expert_fwd(xs, one, [w1], [w3], [w2])
            d_o = O.dispatch(dy, perm[rs], wl.k, row_scale=tw)
            dxp, _, _, _ = O.expert_bwd(xs, h1, h3, d_o, one, [w1], [w3], [w2])
            rs_t = torch.from_numpy(rs).cuda()
            for name, got, ref in (("h1", buf.h1, h1), ("h3", buf.h3, h3), ("o", buf.o, o), ("dxp", buf.dxp, dxp)):
                worst.add(name, host(got[rs_t]), ref)
            # (b) sampled hidden units, all rows of the expert: columns of dW1/dW3, rows of dW2
            J = np.sort(rng.choice(wl.f, size=SAMPLE_UNITS, replace=False))
            xe = x[perm[lo:hi] // wl.k].astype(np.float64)
            one = np.array([0, n], dtype=np.int32)
            h1j, h3j, _, _ = O.expert_fwd(xe, one, [w1[:, J]], [w3[:, J]], [w2[J, :]])
            d_oe = O.dispatch(dy, perm[lo:hi], wl.k, row_scale=tw)
            _, dw1j, dw3j, dw2j = O.expert_bwd(xe, h1j, h3j, d_oe, one, [w1[:, J]], [w3[:, J]], [w2[J, :]])
            Jt = torch.from_numpy(J).cuda()
            for name, got, ref in (("dw1", buf.dw1[e][:, Jt], dw1j[0]), ("dw3", buf.dw3[e][:, Jt], dw3j[0]),
                                   ("dw2", buf.dw2[e][Jt, :], dw2j[0])):
                worst.add(name, host(got), ref)
            print(f"  expert {e}: {len(rs)} of {n} rows and {SAMPLE_UNITS} hidden units checked ({time.time() - t0:.1f}s)", flush=True)
    worst.report()
    bad = {k: v for k, v in worst.mx.items() if not v < tol}
    assert not bad, bad
    bad = {k: v for k, v in worst.l2.items() if not v < tol}
    assert not bad, f"relative l2 error: {bad}"
