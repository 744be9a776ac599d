"""Independent brute-force evaluation of the MoE layer, used only to pin the oracle.

It shares nothing with oracle/: there is no sort, no permutation and no expert-ordered
buffer here.  An expert is selected for a token iff fewer than k experts beat it (higher
logit, or equal logit and lower index) -- a rank count straight from the definition of
"the k experts with the highest scores" in the paper's MoE background section.  The layer
output is then every expert evaluated densely on every token, times a [T,E] matrix of
gate weights that is zero outside the selection and outside the local slice.
"""
import math

import numpy as np
import torch


def selection_mask(logits, k):
    """[T,E] bool via rank counting (pure definition, O(T*E*E))."""
    l = np.asarray(logits, dtype=np.float32)
    T, E = l.shape
    idx = np.arange(E)
    beats = (l[:, None, :] > l[:, :, None]) | ((l[:, None, :] == l[:, :, None]) & (idx[None, None, :] < idx[None, :, None]))
    rank = beats.sum(axis=2)            # rank[t,e] = number of experts that beat e
    return rank < k, rank


def gate_matrix(logits, k, gate_mode):
    """[T,E] float64 gate weights, zero where not selected."""
    mask, _ = selection_mask(logits, k)
    l = np.asarray(logits, dtype=np.float32).astype(np.float64)
    T, E = l.shape
    G = np.zeros((T, E))
    for t in range(T):
        sel = np.nonzero(mask[t])[0]
        if gate_mode == 0:      # softmax over all experts, renormalised over the selection
            p = np.array([math.exp(v - l[t].max()) for v in l[t]])
            p = p / p.sum()
            G[t, sel] = p[sel] / p[sel].sum()
        elif gate_mode == 2:    # plain softmax probability
            p = np.array([math.exp(v - l[t].max()) for v in l[t]])
            G[t, sel] = (p / p.sum())[sel]
        elif gate_mode == 1:    # logistic scores renormalised over the selection
            s = np.array([1.0 / (1.0 + math.exp(-v)) for v in l[t]])
            G[t, sel] = s[sel] / s[sel].sum()
        else:
            raise ValueError
    return G


def dense_layer_torch(x, G_local, w1, w3, w2):
    """y = sum_e G[:,e] * FFN_e(x) over local experts, torch float64 (autograd-capable).
    G_local [T,e_cnt]; w1,w3 [e_cnt,d,f]; w2 [e_cnt,f,d]."""
    y = torch.zeros_like(x)
    for e in range(w1.shape[0]):
        h = torch.nn.functional.silu(x @ w1[e]) * (x @ w3[e])
        y = y + G_local[:, e:e + 1] * (h @ w2[e])
    return y
