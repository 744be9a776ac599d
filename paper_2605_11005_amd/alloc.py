"""ctypes binding of include/moe_alloc.h (host-only worker-allocation tool).  Marshalling only."""
from __future__ import annotations

import ctypes

from .binding import MoeError, load_library


class Model(ctypes.Structure):
    _fields_ = [("C_a", ctypes.c_double), ("C_f", ctypes.c_double), ("V", ctypes.c_double), ("P", ctypes.c_double),
                ("B", ctypes.c_double)]


PROFILE_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_void_p)
EXPORTS = ("moe_alloc_costs", "moe_alloc_eval", "moe_alloc_seed", "moe_alloc_refine", "moe_alloc_group_layers",
           "moe_alloc_bubbles")


def _lib():
    lib = load_library()
    if not getattr(lib, "_alloc_ready", False):
        d, i, dp, ip = ctypes.c_double, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)
        mp = ctypes.POINTER(Model)
        lib.moe_alloc_costs.argtypes = [d, d, d, d, d, d, i, i, dp, dp, dp, dp, dp]
        lib.moe_alloc_eval.argtypes = [mp, i, i, i, i, dp, dp, dp, dp]
        lib.moe_alloc_seed.argtypes = [mp, i, i, d, ip, ip, dp, ip]
        lib.moe_alloc_refine.argtypes = [i, i, i, i, i, ip, ip, PROFILE_FN, ctypes.c_void_p, ip, ip, dp]
        lib.moe_alloc_group_layers.argtypes = [i, i, i, ip, i, ip]
        lib.moe_alloc_bubbles.argtypes = [i, i, i, d, d, d, d, d, dp, dp]
        for n in EXPORTS:
            getattr(lib, n).restype = i
        lib._alloc_ready = True
    return lib


def _ok(rc, name):
    if rc != 0:
        raise MoeError(f"{name}: invalid argument")


def costs(b, S, H, g, k, D_e, n_mat=2, bytes_per_elem=2):
    out = [ctypes.c_double() for _ in range(5)]
    _ok(_lib().moe_alloc_costs(b, S, H, g, k, D_e, n_mat, bytes_per_elem, *[ctypes.byref(o) for o in out]), "moe_alloc_costs")
    return dict(zip(("C_a", "C_f", "V", "I_attn", "I_ffn"), (o.value for o in out)))


def _model(m):
    return Model(m["C_a"], m["C_f"], m["V"], m["P"], m["B"])


def evaluate(model, W, M_tot, M, M_a):
    out = [ctypes.c_double() for _ in range(4)]
    _ok(_lib().moe_alloc_eval(ctypes.byref(_model(model)), W, M_tot, M, M_a, *[ctypes.byref(o) for o in out]), "moe_alloc_eval")
    return dict(zip(("T_a", "T_f", "U_a", "U_f"), (o.value for o in out)))


def seed(model, W, M_tot, eps=0.0):
    M, Ma, n = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    T = ctypes.c_double()
    _ok(_lib().moe_alloc_seed(ctypes.byref(_model(model)), W, M_tot, eps, ctypes.byref(M), ctypes.byref(Ma), ctypes.byref(T),
                              ctypes.byref(n)), "moe_alloc_seed")
    return dict(M=M.value, M_a=Ma.value, T_star=T.value, n_candidates=n.value)


def refine(W, M_tot, M0, Ma0, dM, dMa, profile):
    K = len(dM)
    arr = ctypes.c_int * max(K, 1)
    cb = PROFILE_FN(lambda m, ma, _u: float(profile(m, ma)))
    M, Ma, T = ctypes.c_int(), ctypes.c_int(), ctypes.c_double()
    _ok(_lib().moe_alloc_refine(W, M_tot, M0, Ma0, K, arr(*dM) if K else arr(0), arr(*dMa) if K else arr(0), cb, None,
                                ctypes.byref(M), ctypes.byref(Ma), ctypes.byref(T)), "moe_alloc_refine")
    return M.value, Ma.value, T.value


def group_layers(L, p, g):
    buf = (ctypes.c_int * max(L, 1))()
    n = ctypes.c_int()
    _ok(_lib().moe_alloc_group_layers(L, p, g, buf, L, ctypes.byref(n)), "moe_alloc_group_layers")
    return list(buf[:n.value])


def bubbles(PP, L, v, T_a, T_f, T_a2a, T_p2p, T_m2n):
    base, af = ctypes.c_double(), ctypes.c_double()
    _ok(_lib().moe_alloc_bubbles(PP, L, v, T_a, T_f, T_a2a, T_p2p, T_m2n, ctypes.byref(base), ctypes.byref(af)), "moe_alloc_bubbles")
    return base.value, af.value
