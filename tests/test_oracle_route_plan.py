"""Pins for oracle.route / oracle.plan / dispatch / combine (CPU only).

Each check compares the oracle with something that is not the oracle: a rank-count brute
force, closed forms from tests/golden, scipy's softmax, and the structural invariants the
dispatch permutation must have (bijection onto local (token,slot) pairs, counts summing
to T*k when every expert is local, identity-expert round trip)."""
import os

import numpy as np
import pytest
from scipy.special import expit, softmax

from oracle import moe_oracle as O
from paper_2605_11005_amd import workloads as W
from tests.bruteforce import gate_matrix, selection_mask

GOLD = os.path.join(os.path.dirname(__file__), "golden", "gate_closed_forms.txt")


def _gold_rows():
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        mode, k, logits, idx, w = line.split()
        rows.append((int(mode), int(k), [float(v) for v in logits.split(",")],
                     [int(v) for v in idx.split(",")], [float(v) for v in w.split(",")]))
    return rows


@pytest.mark.parametrize("mode,k,logits,idx,w", _gold_rows())
def test_route_closed_forms(mode, k, logits, idx, w):
    l = np.array([logits], dtype=np.float32)
    ti, tw, cnt = O.route(l, k, mode, 0, l.shape[1])
    assert ti[0].tolist() == idx
    np.testing.assert_allclose(tw[0], w, rtol=0, atol=2e-7)   # logits are fp32-rounded
    assert cnt.sum() == k


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("T,E,k", [(64, 8, 2), (48, 32, 8), (16, 5, 5), (33, 7, 1)])
def test_route_vs_rank_count(mode, T, E, k):
    rng = np.random.default_rng(T * 1000 + E * 10 + k)
    l = rng.standard_normal((T, E)).astype(np.float32)
    l[::3] = np.round(l[::3])            # plenty of exact ties
    l[1, :] = 0.25
    ti, tw, cnt = O.route(l, k, mode, 0, E)
    mask, rank = selection_mask(l, k)
    G = gate_matrix(l, k, mode)
    for t in range(T):
        assert sorted(ti[t].tolist()) == np.nonzero(mask[t])[0].tolist()
        assert [rank[t, e] for e in ti[t]] == list(range(k))      # slot j = j-th best
        np.testing.assert_allclose(tw[t], G[t, ti[t]], rtol=1e-12, atol=1e-15)
    assert cnt.sum() == T * k
    assert cnt.tolist() == mask.sum(axis=0).tolist()


def test_route_library_special_cases():
    rng = np.random.default_rng(5)
    l = rng.standard_normal((20, 6)).astype(np.float32)
    # k = E, plain softmax == scipy softmax in sorted order
    ti, tw, _ = O.route(l, 6, O.GATE_SOFTMAX, 0, 6)
    p = softmax(l.astype(np.float64), axis=1)
    np.testing.assert_allclose(tw, np.take_along_axis(p, ti.astype(np.int64), 1), rtol=1e-12)
    # softmax-renorm with k=2 == logistic of the logit gap
    ti, tw, _ = O.route(l, 2, O.GATE_SOFTMAX_RENORM, 0, 6)
    s = np.sort(l.astype(np.float64), axis=1)
    np.testing.assert_allclose(tw[:, 0], expit(s[:, -1] - s[:, -2]), rtol=1e-12)
    # renormalised modes sum to one, all weights positive
    for mode in (0, 1):
        _, tw, _ = O.route(l, 3, mode, 0, 6)
        np.testing.assert_allclose(tw.sum(1), 1.0, rtol=1e-12)
        assert (tw > 0).all()
    # sigmoid renorm == expit / sum
    ti, tw, _ = O.route(l, 3, O.GATE_SIGMOID_RENORM, 0, 6)
    s = expit(np.take_along_axis(l.astype(np.float64), ti.astype(np.int64), 1))
    np.testing.assert_allclose(tw, s / s.sum(1, keepdims=True), rtol=1e-12)


def test_route_local_counts_partition():
    rng = np.random.default_rng(11)
    T, E, k = 200, 24, 4
    l = rng.standard_normal((T, E)).astype(np.float32)
    total = 0
    for e_lo in range(0, E, 8):
        ti, _, cnt = O.route(l, k, 0, e_lo, 8)
        assert cnt.tolist() == [(ti == e_lo + e).sum() for e in range(8)]
        total += cnt.sum()
    assert total == T * k


@pytest.mark.parametrize("e_lo,e_cnt", [(0, 16), (4, 5), (15, 1), (0, 1)])
def test_plan_is_the_stable_bijection(e_lo, e_cnt):
    rng = np.random.default_rng(e_lo * 7 + e_cnt)
    T, E, k = 300, 16, 3
    l = rng.standard_normal((T, E)).astype(np.float32)
    ti, _, cnt = O.route(l, k, 0, e_lo, e_cnt)
    off, perm, inv = O.plan(ti, e_lo, e_cnt)
    flat = ti.reshape(-1)
    local = (flat >= e_lo) & (flat < e_lo + e_cnt)
    R = int(local.sum())
    assert off[0] == 0 and off[-1] == R and len(perm) == R
    assert np.diff(off).tolist() == cnt.tolist()
    assert off.tolist() == np.concatenate([[0], np.cumsum(cnt)]).tolist()
    # bijection onto the local slots
    assert sorted(perm.tolist()) == np.nonzero(local)[0].tolist()
    assert (inv.reshape(-1)[perm] == np.arange(R)).all()
    assert (inv.reshape(-1)[~local] == -1).all()
    assert (perm[inv.reshape(-1)[local]] == np.nonzero(local)[0]).all()
    for e in range(e_cnt):
        seg = perm[off[e]:off[e + 1]]
        assert (flat[seg] == e_lo + e).all()                 # right expert
        assert (np.diff(seg) > 0).all()                      # ascending slot = stable
    if e_cnt == E:
        assert cnt.sum() == T * k


def test_plan_degenerate_shapes():
    ti = np.zeros((0, 2), dtype=np.int32)
    off, perm, inv = O.plan(ti, 0, 4)
    assert off.tolist() == [0] * 5 and perm.size == 0 and inv.shape == (0, 2)
    ti = np.array([[3, 1], [3, 2]], dtype=np.int32)          # expert 0 empty, expert 3 twice
    off, perm, inv = O.plan(ti, 0, 4)
    assert off.tolist() == [0, 0, 1, 2, 4]
    assert perm.tolist() == [1, 3, 0, 2]
    assert inv.tolist() == [[2, 0], [3, 1]]
    off, perm, inv = O.plan(ti, 0, 2)                        # only experts 0,1 local
    assert off.tolist() == [0, 0, 1] and perm.tolist() == [1] and inv.tolist() == [[-1, 0], [-1, -1]]


@pytest.mark.parametrize("e_lo,e_cnt", [(0, 8), (2, 3)])
def test_identity_expert_round_trip(e_lo, e_cnt):
    """combine(dispatch(x)) with identity experts = x[t] * (sum of the token's local gates)."""
    rng = np.random.default_rng(3)
    T, E, k, d = 120, 8, 3, 16
    x = rng.standard_normal((T, d))
    l = rng.standard_normal((T, E)).astype(np.float32)
    ti, tw, _ = O.route(l, k, 1, e_lo, e_cnt)
    off, perm, inv = O.plan(ti, e_lo, e_cnt)
    xp = O.dispatch(x, perm, k)
    for r in range(len(perm)):                               # row r holds its token
        assert (xp[r] == x[perm[r] // k]).all()
    local = (ti >= e_lo) & (ti < e_lo + e_cnt)
    y = O.combine(xp, inv, tw)
    np.testing.assert_allclose(y, x * (tw * local).sum(1, keepdims=True), rtol=1e-12, atol=1e-14)
    y1 = O.combine(xp, inv, None)
    np.testing.assert_allclose(y1, x * local.sum(1, keepdims=True), rtol=1e-12, atol=1e-14)
    # scaled dispatch (backward of combine): row r = gate * dy
    xs = O.dispatch(x, perm, k, row_scale=tw)
    np.testing.assert_allclose(xs, xp * tw.reshape(-1)[perm][:, None], rtol=1e-15)
    # dispatch and unweighted combine are adjoint linear maps
    g = rng.standard_normal(xp.shape)
    assert abs((xp * g).sum() - (x * O.combine(g, inv, None)).sum()) < 1e-9


def test_workload_generators_shape_popularity():
    """Input-recipe sanity (host logic): Zipf slice share and the skew construction."""
    wl = W.DSV3.scaled(T=4096, d=8, f=8)
    l = W.router_logits(wl)
    ti, tw, cnt = O.route(l, wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt)
    rank = W.expert_rank(wl)
    pop = 1.0 / rank
    share = pop[: wl.e_cnt].sum() / pop.sum()
    assert 0.3 * share < cnt.sum() / (wl.T * wl.k) < 3 * share
    sk = W.SKEW.scaled(T=8192, d=8, f=8)
    l = W.router_logits(sk)
    ti, tw, cnt = O.route(l, sk.k, sk.gate_mode, sk.e_lo, sk.e_cnt)
    hot, empty, cold = W.skew_roles(sk)
    assert all(cnt[e - sk.e_lo] == 0 for e in empty)
    frac_hot = sum(cnt[e - sk.e_lo] for e in hot) / cnt.sum()
    assert 0.45 < frac_hot < 0.55
    assert 0.9 < cnt.sum() / sk.T < 1.1
    # bf16 rounding helper: round-to-nearest-even on the 16 dropped bits
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.14159], dtype=np.float32)
    b = W.bf16_value(W.bf16_bits(a))
    assert b.tolist()[:4] == [1.0, 1.0, 1.015625, -2.5]
    assert abs(b[4] - 3.14159) < 2 ** -7
