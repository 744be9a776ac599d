"""Pins for the oracle's trainable-gate functions (router GEMM, gate gradient, gradient through
the gate weights): torch autograd in float64 on the dense all-experts-then-mask form with a
differentiable gate matrix whose selection mask comes from the rank-count brute force, plus
central finite differences and closed-form special cases.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from tests.bruteforce import dense_layer_torch, selection_mask


def _setup(seed, T=24, d=10, E=6, k=3, f=7, e_lo=0, e_cnt=None):
    rng = np.random.default_rng(seed)
    e_cnt = E - e_lo if e_cnt is None else e_cnt
    return dict(x=rng.standard_normal((T, d)), wr=rng.standard_normal((d, E)) / np.sqrt(d),
                w1=rng.standard_normal((e_cnt, d, f)) / np.sqrt(d), w3=rng.standard_normal((e_cnt, d, f)) / np.sqrt(d),
                w2=rng.standard_normal((e_cnt, f, d)) / np.sqrt(f), dy=rng.standard_normal((T, d)), k=k, e_lo=e_lo, e_cnt=e_cnt)


def _torch_gate(l, mask, mode):
    m = torch.tensor(mask, dtype=torch.float64)
    if mode == 0:
        p = torch.softmax(l, dim=1) * m
        return p / p.sum(dim=1, keepdim=True)
    if mode == 1:
        s = torch.sigmoid(l) * m
        return s / s.sum(dim=1, keepdim=True)
    return torch.softmax(l, dim=1) * m


def _autograd(p, mode, logits32):
    """Loss <dy, y> with y the dense-then-mask layer and gates a differentiable function of x Wr.
    The forward uses the same float32-rounded logits the oracle routes on (selection identical);
    gradients flow through the unrounded product."""
    mask, _ = selection_mask(logits32, p["k"])
    x = torch.tensor(p["x"], requires_grad=True)
    wr = torch.tensor(p["wr"], requires_grad=True)
    l = x @ wr
    G = _torch_gate(l, mask, mode)[:, p["e_lo"]:p["e_lo"] + p["e_cnt"]]
    y = dense_layer_torch(x, G, torch.tensor(p["w1"]), torch.tensor(p["w3"]), torch.tensor(p["w2"]))
    (y * torch.tensor(p["dy"])).sum().backward()
    return y.detach().numpy(), x.grad.numpy(), wr.grad.numpy()


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("e_lo,e_cnt", [(0, 6), (2, 3)])
def test_router_gradients_match_autograd(mode, e_lo, e_cnt):
    p = _setup(10 + mode, e_lo=e_lo, e_cnt=e_cnt)
    logits = O.router_logits(p["x"], p["wr"])
    assert logits.dtype == np.float32
    np.testing.assert_allclose(logits, p["x"] @ p["wr"], rtol=1e-6, atol=1e-6)
    fw = O.layer_fwd(p["x"], logits, p["k"], mode, e_lo, e_cnt, p["w1"], p["w3"], p["w2"])
    bw = O.layer_bwd(fw, p["dy"], p["k"], p["w1"], p["w3"], p["w2"])
    dg = O.gate_grad(p["dy"], fw["o"], fw["inv"])
    dl = O.gate_bwd(logits, fw["topk_idx"], dg, mode)
    dwr, dx_r = O.router_bwd(p["x"], p["wr"], dl)
    y, dx_ref, dwr_ref = _autograd(p, mode, logits)
    # float32 rounding of the logits perturbs the forward at the 1e-7 level only
    np.testing.assert_allclose(fw["y"], y, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(dwr, dwr_ref, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(bw["dx"] + dx_r, dx_ref, rtol=1e-5, atol=1e-6)


def test_gate_grad_definition_and_nonlocal_slots():
    p = _setup(3, e_lo=1, e_cnt=2)
    logits = O.router_logits(p["x"], p["wr"])
    fw = O.layer_fwd(p["x"], logits, p["k"], 0, 1, 2, p["w1"], p["w3"], p["w2"])
    dg = O.gate_grad(p["dy"], fw["o"], fw["inv"])
    for t in range(p["x"].shape[0]):
        for j in range(p["k"]):
            r = fw["inv"][t, j]
            want = 0.0 if r < 0 else float(p["dy"][t] @ fw["o"][r])
            assert abs(dg[t, j] - want) < 1e-12
    # <dy, y> is linear in the gate weights: y(g + h) - y(g) = <dg, h>
    h = np.random.default_rng(0).standard_normal(dg.shape)
    y0 = O.combine(fw["o"], fw["inv"], fw["topk_w"]); y1 = O.combine(fw["o"], fw["inv"], fw["topk_w"] + h)
    assert abs(((y1 - y0) * p["dy"]).sum() - (dg * h).sum()) < 1e-9


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_gate_bwd_by_finite_differences_and_invariants(mode):
    rng = np.random.default_rng(5 + mode)
    T, E, k = 9, 7, 3
    l = rng.standard_normal((T, E)).astype(np.float32)
    idx, w, _ = O.route(l, k, mode, 0, E)
    dg = rng.standard_normal((T, k))
    dl = O.gate_bwd(l, idx, dg, mode)
    # finite differences of sum(dg * w(l)) with the selection held fixed
    def weights(lv):
        lv = lv.astype(np.float64)
        sel = np.take_along_axis(lv, idx.astype(np.int64), 1)
        if mode == 0:
            e = np.exp(sel); return e / e.sum(1, keepdims=True)
        if mode == 1:
            s = 1 / (1 + np.exp(-sel)); return s / s.sum(1, keepdims=True)
        p = np.exp(lv) / np.exp(lv).sum(1, keepdims=True)
        return np.take_along_axis(p, idx.astype(np.int64), 1)
    h = 1e-6
    for _ in range(5):
        direction = rng.standard_normal((T, E))
        fd = ((weights(l.astype(np.float64) + h * direction) * dg).sum() - (weights(l.astype(np.float64) - h * direction) * dg).sum()) / (2 * h)
        assert abs(fd - (dl * direction).sum()) < 1e-7
    if mode in (0, 1):
        # renormalised weights sum to one: a constant dg has no effect; unselected logits get no gradient
        assert np.abs(O.gate_bwd(l, idx, np.ones((T, k)), mode)).max() < 1e-12
        mask = np.zeros((T, E), bool); np.put_along_axis(mask, idx.astype(np.int64), True, 1)
        assert not dl[~mask].any()
    if mode in (0, 2):
        np.testing.assert_allclose(dl.sum(1), 0.0, atol=1e-12)      # softmax: shift invariance


def test_router_bwd_is_the_adjoint_of_the_router_gemm():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((11, 5)); wr = rng.standard_normal((5, 4)); dl = rng.standard_normal((11, 4))
    dwr, dx = O.router_bwd(x, wr, dl)
    dW = rng.standard_normal(wr.shape); dX = rng.standard_normal(x.shape)
    assert abs(((x @ dW) * dl).sum() - (dwr * dW).sum()) < 1e-10
    assert abs(((dX @ wr) * dl).sum() - (dx * dX).sum()) < 1e-10
