"""Pins for the oracle's expert FFNs, whole layer and gradients (CPU only).

Compared against: a dense SwiGLU MLP written with torch library ops (E=1, k=1), the
dense all-experts-then-mask brute force, torch autograd in float64 on that brute force,
and central finite differences.  Planted-mistake checks at the end show that a dropped
term, a swapped W1/W3 or a transposed operand would be caught."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2605_11005_amd import workloads as W
from tests.bruteforce import dense_layer_torch, gate_matrix


def _tiny(seed=0, T=40, d=12, E=6, k=2, f=10, e_lo=0, e_cnt=None, mode=0):
    rng = np.random.default_rng(seed)
    e_cnt = E - e_lo if e_cnt is None else e_cnt
    x = rng.standard_normal((T, d))
    l = rng.standard_normal((T, E)).astype(np.float32)
    w1 = rng.standard_normal((e_cnt, d, f)) / np.sqrt(d)
    w3 = rng.standard_normal((e_cnt, d, f)) / np.sqrt(d)
    w2 = rng.standard_normal((e_cnt, f, d)) / np.sqrt(f)
    dy = rng.standard_normal((T, d))
    return dict(x=x, l=l, w1=w1, w3=w3, w2=w2, dy=dy, k=k, mode=mode, e_lo=e_lo, e_cnt=e_cnt)


def _torch_ref(p):
    """Brute force + autograd: returns y, dx, dw1, dw3, dw2 as numpy float64."""
    G = gate_matrix(p["l"], p["k"], p["mode"])[:, p["e_lo"]:p["e_lo"] + p["e_cnt"]]
    tx = torch.tensor(p["x"], dtype=torch.float64, requires_grad=True)
    t1 = torch.tensor(p["w1"], dtype=torch.float64, requires_grad=True)
    t3 = torch.tensor(p["w3"], dtype=torch.float64, requires_grad=True)
    t2 = torch.tensor(p["w2"], dtype=torch.float64, requires_grad=True)
    y = dense_layer_torch(tx, torch.tensor(G), t1, t3, t2)
    (y * torch.tensor(p["dy"])).sum().backward()
    return [v.detach().numpy() for v in (y, tx.grad, t1.grad, t3.grad, t2.grad)]


def _oracle(p):
    fw = O.layer_fwd(p["x"], p["l"], p["k"], p["mode"], p["e_lo"], p["e_cnt"], p["w1"], p["w3"], p["w2"])
    bw = O.layer_bwd(fw, p["dy"], p["k"], p["w1"], p["w3"], p["w2"])
    return fw, bw


def test_single_expert_is_a_dense_swiglu_mlp():
    p = _tiny(seed=1, E=1, k=1, T=17)
    fw, _ = _oracle(p)
    x = torch.tensor(p["x"])
    ref = (torch.nn.functional.silu(x @ torch.tensor(p["w1"][0])) * (x @ torch.tensor(p["w3"][0]))) @ torch.tensor(p["w2"][0])
    np.testing.assert_allclose(fw["y"], ref.numpy(), rtol=1e-12, atol=1e-13)   # gate weight is 1
    assert fw["perm"].tolist() == list(range(17))


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("e_lo,e_cnt", [(0, 6), (1, 3), (5, 1)])
def test_layer_matches_dense_then_mask(mode, e_lo, e_cnt):
    p = _tiny(seed=2 + mode, e_lo=e_lo, e_cnt=e_cnt, mode=mode, k=3)
    fw, bw = _oracle(p)
    y, dx, dw1, dw3, dw2 = _torch_ref(p)
    np.testing.assert_allclose(fw["y"], y, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(bw["dx"], dx, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw["dw1"], dw1, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw["dw3"], dw3, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw["dw2"], dw2, rtol=1e-10, atol=1e-12)


def test_tiny_headline_config_matches_dense_then_mask():
    wl = W.TINY.scaled(T=64)
    x = W.tokens(wl)
    p = dict(x=x.astype(np.float64), l=W.router_logits(wl, x), k=wl.k, mode=wl.gate_mode, e_lo=0, e_cnt=wl.E,
             dy=W.out_grad(wl).astype(np.float64))
    w1, w3, w2 = W.all_expert_weights(wl)
    p.update(w1=w1.astype(np.float64), w3=w3.astype(np.float64), w2=w2.astype(np.float64))
    fw, bw = _oracle(p)
    y, dx, dw1, dw3, dw2 = _torch_ref(p)
    np.testing.assert_allclose(fw["y"], y, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw["dx"], dx, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw["dw2"], dw2, rtol=1e-10, atol=1e-12)


def test_gradients_by_central_differences():
    p = _tiny(seed=9, T=12, d=6, E=4, k=2, f=5)
    fw, bw = _oracle(p)
    rng = np.random.default_rng(0)

    def obj(q):
        return (O.layer_fwd(q["x"], q["l"], q["k"], q["mode"], 0, 4, q["w1"], q["w3"], q["w2"])["y"] * q["dy"]).sum()

    for name, grad in (("x", bw["dx"]), ("w1", bw["dw1"]), ("w3", bw["dw3"]), ("w2", bw["dw2"])):
        direction = rng.standard_normal(p[name].shape)
        h = 1e-6
        qp = dict(p); qm = dict(p)
        qp[name] = p[name] + h * direction
        qm[name] = p[name] - h * direction
        fd = (obj(qp) - obj(qm)) / (2 * h)
        an = (grad * direction).sum()
        assert abs(fd - an) < 1e-6 * max(1.0, abs(an)), name


def test_empty_expert_and_linearity():
    p = _tiny(seed=4, T=9, E=6, k=1)
    p["l"][:, 2] = -50.0                                      # expert 2 never chosen
    fw, bw = _oracle(p)
    assert fw["counts"][2] == 0
    assert not bw["dw1"][2].any() and not bw["dw3"][2].any() and not bw["dw2"][2].any()
    q = dict(p); q["dy"] = 3.0 * p["dy"]
    _, bw3 = _oracle(q)
    np.testing.assert_allclose(bw3["dx"], 3.0 * bw["dx"], rtol=1e-12)
    np.testing.assert_allclose(bw3["dw2"], 3.0 * bw["dw2"], rtol=1e-12)


def test_token_permutation_equivariance():
    p = _tiny(seed=6, T=30)
    fw, _ = _oracle(p)
    sh = np.random.default_rng(1).permutation(30)
    q = dict(p); q["x"] = p["x"][sh]; q["l"] = p["l"][sh]; q["dy"] = p["dy"][sh]
    fw2, _ = _oracle(q)
    np.testing.assert_allclose(fw2["y"], fw["y"][sh], rtol=1e-12, atol=1e-14)


def test_planted_mistakes_are_caught():
    """A wrong sign/index/transposition in the expert math must fail the dense pin."""
    p = _tiny(seed=7)
    y, dx, dw1, dw3, dw2 = _torch_ref(p)
    fw, bw = _oracle(p)
    # swapped gate/linear branch
    bad = O.layer_fwd(p["x"], p["l"], p["k"], p["mode"], 0, 6, p["w3"], p["w1"], p["w2"])["y"]
    assert np.abs(bad - y).max() > 1e-3
    # dropped silu' term: dH1 without the z*(1-sig) part
    z = fw["h1"]; sig = 1 / (1 + np.exp(-z))
    dA = np.zeros_like(z)
    for e in range(6):
        lo, hi = fw["offsets"][e], fw["offsets"][e + 1]
        dA[lo:hi] = bw["d_o"][lo:hi] @ p["w2"][e].T
    wrong_dH1 = dA * fw["h3"] * sig
    right_dH1 = dA * fw["h3"] * sig * (1 + z * (1 - sig))
    assert np.abs(wrong_dH1 - right_dH1).max() > 1e-3
    e = int(np.argmax(fw["counts"])); lo, hi = fw["offsets"][e], fw["offsets"][e + 1]
    np.testing.assert_allclose(fw["xp"][lo:hi].T @ right_dH1[lo:hi], dw1[e], rtol=1e-9, atol=1e-11)
    assert np.abs(fw["xp"][lo:hi].T @ wrong_dH1[lo:hi] - dw1[e]).max() > 1e-3
    # unweighted combine instead of gate-weighted
    assert np.abs(O.combine(fw["o"], fw["inv"], None) - y).max() > 1e-3
