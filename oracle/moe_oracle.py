"""CPU oracle for one GPU's share of a Mixture-of-Experts expert layer.  TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file;
the product (the HIP library and its binding) never does, and shares no code with it.

What it computes is the plain definition from the paper's background section on MoE
structure: a gate picks, per token, the top-k experts with the highest scores; the
outputs of those experts are reduced by a weighted sum.  One FFN-group GPU holds a
contiguous slice of the experts (expert parallelism, background section on
distributed training) and contributes the partial sum over its local experts:

    y_t = sum_{e in TopK(t), e local} g_{t,e} * FFN_e(x_t)
    FFN_e(x) = (silu(x W1_e) * (x W3_e)) W2_e             (SwiGLU, no biases)

The expert work is the grouped GEMM over expert-contiguous rows that the paper's
resource-allocation section counts as the expert FLOPs; its dispatch/combine are the
shuffles between micro-batch order and expert order described in the introduction.

Everything is numpy in float64 (a library matmul is used as a step; no blocking,
fusion or reordering).  Integer artefacts are int32 and are unique given the
readings below, so they can be compared bit for bit.

Readings where the paper is silent:
  * ranking is on the raw fp32 logits (softmax and sigmoid are increasing, so the
    selected set is the same); equal logits -> lower expert index first; +0 == -0.
  * slot j of a token is its j-th best expert.
  * gate weights: SOFTMAX_RENORM p_j / sum_topk p (p = softmax over all E);
    SIGMOID_RENORM s_j / sum_topk s (s = logistic); SOFTMAX p_j (no renormalisation).
  * dropless: every (token, slot) pair with a local expert gets a row.
  * rows are ordered by (local expert, flat slot s = t*k + j).
  * inv[t,j] = row of slot (t,j), or -1 if its expert is not local.
  * the gate multiplies after the down projection, inside combine; combine adds the
    slots in ascending j.
  * dX is the gradient through the expert path only (logits are an input).

Every function here is pinned by tests/test_oracle_*.py against something that is not
this file: a rank-count brute force, closed forms, a dense all-experts-then-mask
evaluation, torch autograd in fp64 and central finite differences.
"""
from __future__ import annotations

import numpy as np

GATE_SOFTMAX_RENORM = 0
GATE_SIGMOID_RENORM = 1
GATE_SOFTMAX = 2


# ------------------------------------------------------------------ route
def route(logits, k, gate_mode, e_lo, e_cnt):
    """Top-k gating.  logits [T,E] fp32.  Returns topk_idx [T,k] int32 (global expert ids,
    slot 0 = best), topk_w [T,k] float64, counts [e_cnt] int32 (rows per local expert)."""
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    assert 1 <= k <= E and 0 <= e_lo and e_lo + e_cnt <= E
    # descending logit, ties by ascending index: a stable sort of the negated values.
    # (-x is exact; +0 and -0 compare equal and so stay in index order.)
    order = np.argsort(-logits, axis=1, kind="stable")
    topk_idx = order[:, :k].astype(np.int32)
    l = logits.astype(np.float64)
    sel = np.take_along_axis(l, topk_idx.astype(np.int64), axis=1)
    if gate_mode == GATE_SOFTMAX_RENORM:
        p = np.exp(l - l.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        ps = np.take_along_axis(p, topk_idx.astype(np.int64), axis=1)
        topk_w = ps / ps.sum(axis=1, keepdims=True)
    elif gate_mode == GATE_SOFTMAX:
        p = np.exp(l - l.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        topk_w = np.take_along_axis(p, topk_idx.astype(np.int64), axis=1)
    elif gate_mode == GATE_SIGMOID_RENORM:
        s = 1.0 / (1.0 + np.exp(-sel))
        topk_w = s / s.sum(axis=1, keepdims=True)
    else:
        raise ValueError("gate_mode")
    counts = np.zeros(e_cnt, dtype=np.int32)
    for e in range(e_cnt):
        counts[e] = np.count_nonzero(topk_idx == e_lo + e)
    return topk_idx, topk_w, counts


# ------------------------------------------------------------------ plan
def plan(topk_idx, e_lo, e_cnt):
    """The permutation from micro-batch order to expert order.
    Returns offsets [e_cnt+1], perm [R] (row -> flat slot), inv [T,k] (slot -> row or -1)."""
    topk_idx = np.asarray(topk_idx)
    T, k = topk_idx.shape
    flat = topk_idx.reshape(-1)
    segs = [np.nonzero(flat == e_lo + e)[0] for e in range(e_cnt)]   # ascending s per expert
    offsets = np.zeros(e_cnt + 1, dtype=np.int32)
    for e in range(e_cnt):
        offsets[e + 1] = offsets[e] + len(segs[e])
    perm = (np.concatenate(segs) if e_cnt else np.zeros(0)).astype(np.int32)
    inv = np.full(T * k, -1, dtype=np.int32)
    for r in range(len(perm)):
        inv[perm[r]] = r
    return offsets, perm, inv.reshape(T, k)


# ------------------------------------------------------------------ dispatch / combine
def dispatch(x, perm, k, row_scale=None):
    """xp[r,:] = x[perm[r] // k, :] (times row_scale at that slot, if given).  float64."""
    x = np.asarray(x, dtype=np.float64)
    perm = np.asarray(perm, dtype=np.int64)
    xp = x[perm // k, :].copy()
    if row_scale is not None:
        xp *= np.asarray(row_scale, dtype=np.float64).reshape(-1)[perm][:, None]
    return xp


def combine(o, inv, topk_w=None):
    """y[t,:] = sum over local slots j (ascending) of topk_w[t,j] * o[inv[t,j], :];
    tokens with no local slot give zeros.  topk_w None -> weight 1."""
    o = np.asarray(o, dtype=np.float64)
    inv = np.asarray(inv)
    T, k = inv.shape
    y = np.zeros((T, o.shape[1]), dtype=np.float64)
    for j in range(k):
        rows = inv[:, j]
        m = rows >= 0
        w = np.ones(T) if topk_w is None else np.asarray(topk_w, dtype=np.float64)[:, j]
        y[m] += w[m, None] * o[rows[m]]
    return y


# ------------------------------------------------------------------ experts
def silu(z):
    return z / (1.0 + np.exp(-z))


def expert_fwd(xp, offsets, w1, w3, w2):
    """Per local expert e, on its rows [offsets[e], offsets[e+1]):
    h1 = xp W1[e], h3 = xp W3[e], a = silu(h1)*h3, o = a W2[e].
    w1/w3/w2 are indexable by local expert (arrays [e_cnt,d,f] / [e_cnt,f,d] or lists)."""
    xp = np.asarray(xp, dtype=np.float64)
    R = int(offsets[-1])
    e_cnt = len(offsets) - 1
    f = np.asarray(w1[0]).shape[1]
    d = xp.shape[1]
    h1 = np.zeros((R, f)); h3 = np.zeros((R, f)); a = np.zeros((R, f)); o = np.zeros((R, d))
    for e in range(e_cnt):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        W1 = np.asarray(w1[e], dtype=np.float64)
        W3 = np.asarray(w3[e], dtype=np.float64)
        W2 = np.asarray(w2[e], dtype=np.float64)
        h1[lo:hi] = xp[lo:hi] @ W1
        h3[lo:hi] = xp[lo:hi] @ W3
        a[lo:hi] = silu(h1[lo:hi]) * h3[lo:hi]
        o[lo:hi] = a[lo:hi] @ W2
    return h1, h3, a, o


def expert_bwd(xp, h1, h3, d_o, offsets, w1, w3, w2):
    """Gradients of <d_o, o> for the expert FFNs.  Returns dxp [R,d], dw1, dw3 [e_cnt,d,f],
    dw2 [e_cnt,f,d]; an expert without rows gets zero weight gradients."""
    xp = np.asarray(xp, dtype=np.float64)
    h1 = np.asarray(h1, dtype=np.float64)
    h3 = np.asarray(h3, dtype=np.float64)
    d_o = np.asarray(d_o, dtype=np.float64)
    e_cnt = len(offsets) - 1
    d = xp.shape[1]
    f = h1.shape[1]
    dxp = np.zeros_like(xp)
    dw1 = np.zeros((e_cnt, d, f)); dw3 = np.zeros((e_cnt, d, f)); dw2 = np.zeros((e_cnt, f, d))
    for e in range(e_cnt):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        W1 = np.asarray(w1[e], dtype=np.float64)
        W3 = np.asarray(w3[e], dtype=np.float64)
        W2 = np.asarray(w2[e], dtype=np.float64)
        z = h1[lo:hi]
        sig = 1.0 / (1.0 + np.exp(-z))
        s = z * sig
        a = s * h3[lo:hi]
        dA = d_o[lo:hi] @ W2.T
        dw2[e] = a.T @ d_o[lo:hi]
        dH1 = dA * h3[lo:hi] * (sig * (1.0 + z * (1.0 - sig)))
        dH3 = dA * s
        dw1[e] = xp[lo:hi].T @ dH1
        dw3[e] = xp[lo:hi].T @ dH3
        dxp[lo:hi] = dH1 @ W1.T + dH3 @ W3.T
    return dxp, dw1, dw3, dw2


# ------------------------------------------------------------------ whole layer
def layer_fwd(x, logits, k, gate_mode, e_lo, e_cnt, w1, w3, w2):
    """route -> plan -> dispatch -> experts -> combine.  Returns a dict of every artefact."""
    topk_idx, topk_w, counts = route(logits, k, gate_mode, e_lo, e_cnt)
    offsets, perm, inv = plan(topk_idx, e_lo, e_cnt)
    xp = dispatch(x, perm, k)
    h1, h3, a, o = expert_fwd(xp, offsets, w1, w3, w2)
    y = combine(o, inv, topk_w)
    return dict(topk_idx=topk_idx, topk_w=topk_w, counts=counts, offsets=offsets, perm=perm,
                inv=inv, xp=xp, h1=h1, h3=h3, a=a, o=o, y=y)


def layer_bwd(fw, dy, k, w1, w3, w2):
    """Backward of layer_fwd for the objective <dy, y>, routing held fixed:
    d_o = gate-scaled dispatch of dy; expert backward; dx = unweighted combine of dxp."""
    d_o = dispatch(dy, fw["perm"], k, row_scale=fw["topk_w"])
    dxp, dw1, dw3, dw2 = expert_bwd(fw["xp"], fw["h1"], fw["h3"], d_o, fw["offsets"], w1, w3, w2)
    dx = combine(dxp, fw["inv"], None)
    return dict(d_o=d_o, dxp=dxp, dw1=dw1, dw3=dw3, dw2=dw2, dx=dx)


# ------------------------------------------------------------------ router (trainable gate)
# The gate is trainable (MoE background section): logits = x Wr, and the loss gradient reaches
# Wr and x through the gate weights.  Selection is held fixed (it is piecewise constant).
def router_logits(x, wr):
    """logits [T,E] = x [T,d] @ Wr [d,E], float64 accumulate, returned as the float32 the router emits."""
    return (np.asarray(x, dtype=np.float64) @ np.asarray(wr, dtype=np.float64)).astype(np.float32)


def gate_grad(dy, o, inv):
    """dg[t,j] = <dy[t], o[inv[t,j]]> for local slots, 0 for slots whose expert is not local
    (y = sum_j g[t,j] * o[inv[t,j]], so this is d<dy,y>/dg)."""
    dy = np.asarray(dy, dtype=np.float64)
    o = np.asarray(o, dtype=np.float64)
    inv = np.asarray(inv)
    T, k = inv.shape
    dg = np.zeros((T, k))
    for j in range(k):
        rows = inv[:, j]
        m = rows >= 0
        dg[m, j] = np.einsum("td,td->t", dy[m], o[rows[m]])
    return dg


def gate_bwd(logits, topk_idx, dg, gate_mode):
    """d<dy,y>/dlogits [T,E] given the complete dg [T,k], selection held fixed."""
    l = np.asarray(logits, dtype=np.float32).astype(np.float64)
    idx = np.asarray(topk_idx).astype(np.int64)
    dg = np.asarray(dg, dtype=np.float64)
    T, E = l.shape
    dl = np.zeros((T, E))
    sel = np.take_along_axis(l, idx, axis=1)
    if gate_mode == GATE_SOFTMAX_RENORM:
        w = np.exp(sel - sel.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)                     # softmax over the selected logits
        d_sel = w * (dg - (w * dg).sum(axis=1, keepdims=True))
        np.put_along_axis(dl, idx, d_sel, axis=1)
    elif gate_mode == GATE_SIGMOID_RENORM:
        s = 1.0 / (1.0 + np.exp(-sel))
        S = s.sum(axis=1, keepdims=True)
        w = s / S
        ds = (dg - (w * dg).sum(axis=1, keepdims=True)) / S
        np.put_along_axis(dl, idx, ds * s * (1.0 - s), axis=1)
    elif gate_mode == GATE_SOFTMAX:
        p = np.exp(l - l.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        ps = np.take_along_axis(p, idx, axis=1)
        inner = (ps * dg).sum(axis=1, keepdims=True)          # sum over selected of p_i dg_i
        dl = -p * inner
        np.put_along_axis(dl, idx, ps * (dg - inner), axis=1)
    else:
        raise ValueError("gate_mode")
    return dl


def router_bwd(x, wr, dlogits):
    """dWr [d,E] = x^T dlogits;  router term of dx [T,d] = dlogits Wr^T."""
    x = np.asarray(x, dtype=np.float64)
    wr = np.asarray(wr, dtype=np.float64)
    dl = np.asarray(dlogits, dtype=np.float64)
    return x.T @ dl, dl @ wr.T
