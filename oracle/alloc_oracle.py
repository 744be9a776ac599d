"""CPU oracle for the worker-allocation tool.  TEST INFRASTRUCTURE (only tests import it).

Written from the paper's section on adaptive worker allocation, independently of the C++ tool:
plain Python, one formula per function, exhaustive search with explicit lists.

  * costs: the roofline paragraph's FLOP and byte counts,
        C_a = b (S H^2 (2 + 2/g) + 4 S^2 H),  C_f = b 2 n_mat k S H D_e,  V = b bytes k S H.
  * stage latencies: T_a = max(C_a/(P M), V/(M_a B)), T_f = max(C_f/(P N), V/(M_f B)).
  * phases 1-2 of the allocation algorithm: scan (M, M_a) with M outer, both ascending; keep the
    running minimum T* of max(T_a, T_f) with the tolerance rule of the algorithm (a strictly
    better split, by more than eps, restarts the candidate list; a split within eps joins it);
    then pick the candidate with the largest score.
    Reading of the tie-break score: the paper says to maximise I_attn + I_ffn among the
    candidates; the model constants C/V do not depend on the split, so the score is taken as the
    two groups' attained fractions of their compute roofs, U_a + U_f with U = C / (P G T):
    min(1, I * NICs * B / (P * GPUs)) per group, i.e. how far the NIC split lifts each group to
    its roof.
  * phase 3: local search on a user-supplied profile function with given perturbations.
  * placement: group g of a component holds layers g, g+p, g+2p, ... below L.
  * warm-up bubbles of the baseline pipeline and of AF-Pipe.
"""
from __future__ import annotations


def costs(b, S, H, g, k, D_e, n_mat=2, bytes_per_elem=2):
    attn = b * (S * H * H * (2 + 2 / g) + 4 * S * S * H)
    ffn = b * (2 * n_mat * k * S * H * D_e)
    vol = b * (bytes_per_elem * k * S * H)
    return dict(C_a=attn, C_f=ffn, V=vol, I_attn=attn / vol, I_ffn=ffn / vol)


def stage_times(model, W, M_tot, M, M_a):
    N, M_f = W - M, M_tot - M_a
    t_a = max(model["C_a"] / (model["P"] * M), model["V"] / (M_a * model["B"]))
    t_f = max(model["C_f"] / (model["P"] * N), model["V"] / (M_f * model["B"]))
    return t_a, t_f


def attained(model, W, M_tot, M, M_a):
    t_a, t_f = stage_times(model, W, M_tot, M, M_a)
    return model["C_a"] / (model["P"] * M * t_a), model["C_f"] / (model["P"] * (W - M) * t_f)


def seed(model, W, M_tot, eps=0.0):
    t_star = float("inf")
    cands = []
    for M in range(1, W):
        for M_a in range(1, M_tot):
            t = max(stage_times(model, W, M_tot, M, M_a))
            if t < t_star - eps:
                t_star = t
                cands = [(M, M_a)]
            elif t <= t_star + eps:
                cands.append((M, M_a))
    scores = [sum(attained(model, W, M_tot, M, M_a)) for (M, M_a) in cands]
    best = max(range(len(cands)), key=lambda i: (scores[i], -i))      # first of the best
    return dict(M=cands[best][0], M_a=cands[best][1], T_star=t_star, candidates=cands)


def refine(W, M_tot, M0, Ma0, dM, dMa, profile):
    m, ma = M0, Ma0
    t = profile(m, ma)
    for a, c in zip(dM, dMa):
        cm = min(max(m + a, 1), W - 1)
        cma = min(max(ma + c, 1), M_tot - 1)
        ct = profile(cm, cma)
        if ct < t:
            m, ma, t = cm, cma, ct
    return m, ma, t


def group_layers(L, p, g):
    return [layer for layer in range(L) if layer % p == g]


def bubbles(PP, L, v, T_a, T_f, T_a2a, T_p2p, T_m2n):
    base = (PP - 1) * (L * (T_a + T_f + 2 * T_a2a) + T_p2p) / v
    af = (PP - 1) * (max(T_a, T_f) + T_m2n) / (2 * v)
    return base, af
