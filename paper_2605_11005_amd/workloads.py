"""Seeded synthetic inputs for the MoE expert layer (shapes only; no method arithmetic).

This module is the one thing the CPU oracle's tests and the HIP path's tests/bench
share: both sides consume exactly the arrays produced here.  It holds nothing of the
method itself (no top-k, no permutation, no FFN) -- only random draws, the logit
recipes that shape expert popularity, and bf16 rounding of *inputs*.

The five workloads take the shapes of the MoE layers the paper trains (its model
table in the evaluation section lists hidden size, expert count, top-k and expert
hidden size) as seen by one FFN-group GPU holding a contiguous slice of experts
(expert parallelism, background section on distributed training).  They stand in
for the paper's pre-training data and checkpoints, which are not available.

Every tensor comes from its own Philox stream keyed by (seed, tensor id, expert),
so a test can materialise a single expert's weights without generating the others.
bf16 workloads are rounded once (round-to-nearest-even) on the host; the rounded
values are what both the oracle (as fp32/fp64) and the GPU (as bf16 bits) see.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
import os

import numpy as np
from numpy.random import Generator, Philox

SEED_BASE = 2605_11005

GATE_SOFTMAX_RENORM = 0
GATE_SIGMOID_RENORM = 1
GATE_SOFTMAX = 2

# tensor ids for the Philox key
_TID = {"x": 1, "router": 2, "bias": 3, "w1": 4, "w3": 5, "w2": 6, "dy": 7, "rank": 8, "route": 9}


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # seed offset; 1..5 are the headline configurations
    T: int                # tokens
    d: int                # hidden size (the paper's H)
    E: int                # experts in the layer
    e_lo: int             # first local expert
    e_cnt: int            # local experts on this GPU
    k: int                # top-k
    f: int                # expert hidden size (the paper's D_e)
    dtype: str            # "f32" or "bf16"
    gate_mode: int
    routing: str          # "router_gemm" | "bias_normal" | "zipf" | "skew"
    zipf_s: float = 0.0
    bias_std: float = 0.0

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    def scaled(self, **kw) -> "Workload":
        """Same recipe at another size (parity tests use reduced shapes)."""
        return replace(self, **kw)


TINY = Workload("tiny-fp32", 1, T=256, d=128, E=8, e_lo=0, e_cnt=8, k=2, f=256,
                dtype="f32", gate_mode=GATE_SOFTMAX_RENORM, routing="router_gemm")
MIXTRAL = Workload("mixtral-like", 2, T=16384, d=4096, E=8, e_lo=0, e_cnt=8, k=2, f=14336,
                   dtype="bf16", gate_mode=GATE_SOFTMAX_RENORM, routing="bias_normal", bias_std=0.5)
QWEN = Workload("qwen-like-share", 3, T=16384, d=2048, E=128, e_lo=0, e_cnt=16, k=8, f=768,
                dtype="bf16", gate_mode=GATE_SOFTMAX_RENORM, routing="zipf", zipf_s=1.1)
DSV3 = Workload("dsv3-like-share", 4, T=32768, d=7168, E=256, e_lo=0, e_cnt=32, k=8, f=2048,
                dtype="bf16", gate_mode=GATE_SIGMOID_RENORM, routing="zipf", zipf_s=1.0)
SKEW = Workload("dsv3-skew", 5, T=32768, d=7168, E=256, e_lo=0, e_cnt=32, k=8, f=2048,
                dtype="bf16", gate_mode=GATE_SIGMOID_RENORM, routing="skew")

CONFIGS = [TINY, MIXTRAL, QWEN, DSV3, SKEW]

# The three models of the paper's model-configuration table (hidden size, experts, top-k, expert
# hidden size) as one GPU's share under 8-way expert parallelism, 16384 tokens per step.
# Hidden sizes 2880 and 1408 are not multiples of the 256-wide GEMM tile: N and M tail tiles.
DSMOE_T2 = Workload("deepseek-moe-share", 6, T=16384, d=2048, E=64, e_lo=0, e_cnt=8, k=4, f=1408,
                    dtype="bf16", gate_mode=GATE_SOFTMAX_RENORM, routing="zipf", zipf_s=1.0)
GPTOSS_T2 = Workload("gpt-oss-share", 7, T=16384, d=2880, E=128, e_lo=0, e_cnt=16, k=4, f=2880,
                     dtype="bf16", gate_mode=GATE_SOFTMAX_RENORM, routing="zipf", zipf_s=1.0)
QWEN3_T2 = Workload("qwen3-share", 8, T=16384, d=4096, E=128, e_lo=0, e_cnt=16, k=8, f=1536,
                    dtype="bf16", gate_mode=GATE_SOFTMAX_RENORM, routing="zipf", zipf_s=1.0)
MODEL_TABLE = [DSMOE_T2, GPTOSS_T2, QWEN3_T2]
BY_NAME = {w.name: w for w in CONFIGS + MODEL_TABLE}


# ----------------------------------------------------------------------------- bf16
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even.  Finite inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_value(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the fp32 values they denote."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_like(wl: Workload, a: np.ndarray) -> np.ndarray:
    """Return `a` as the fp32 array both sides consume (bf16-rounded if wl is bf16)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_value(bf16_bits(a)) if wl.dtype == "bf16" else a


# ----------------------------------------------------------------------------- draws
def _rng(wl: Workload, tensor: str, sub: int = 0) -> Generator:
    return Generator(Philox(key=[wl.seed, (_TID[tensor] << 32) | sub]))


def _normal(wl, tensor, shape, std, sub=0):
    a = _rng(wl, tensor, sub).standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return a


def tokens(wl: Workload) -> np.ndarray:
    """x [T,d] ~ N(0,1)."""
    return round_like(wl, _normal(wl, "x", (wl.T, wl.d), 1.0))


def out_grad(wl: Workload) -> np.ndarray:
    """dY [T,d] ~ N(0,1)."""
    return round_like(wl, _normal(wl, "dy", (wl.T, wl.d), 1.0))


def expert_weights(wl: Workload, e_local: int):
    """(W1[d,f], W3[d,f], W2[f,d]) of local expert e_local; W1,W3 ~ N(0,1/d), W2 ~ N(0,1/f)
    (second argument = variance)."""
    e = wl.e_lo + e_local
    w1 = round_like(wl, _normal(wl, "w1", (wl.d, wl.f), wl.d ** -0.5, e))
    w3 = round_like(wl, _normal(wl, "w3", (wl.d, wl.f), wl.d ** -0.5, e))
    w2 = round_like(wl, _normal(wl, "w2", (wl.f, wl.d), wl.f ** -0.5, e))
    return w1, w3, w2


def all_expert_weights(wl: Workload, out_bits: bool = False, threads: int | None = None):
    """Stacked local weights W1,W3 [e_cnt,d,f], W2 [e_cnt,f,d].

    out_bits=True returns bf16 bit patterns (uint16) instead of fp32 values, which
    halves host memory at the large shapes; only valid for bf16 workloads."""
    if out_bits and wl.dtype != "bf16":
        raise ValueError("bit output is for bf16 workloads")
    dt = np.uint16 if out_bits else np.float32
    w1 = np.empty((wl.e_cnt, wl.d, wl.f), dt)
    w3 = np.empty((wl.e_cnt, wl.d, wl.f), dt)
    w2 = np.empty((wl.e_cnt, wl.f, wl.d), dt)

    def one(e):
        a, b, c = expert_weights(wl, e)
        if out_bits:
            a, b, c = bf16_bits(a), bf16_bits(b), bf16_bits(c)
        w1[e], w3[e], w2[e] = a, b, c

    n = threads or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(n) as ex:
        list(ex.map(one, range(wl.e_cnt)))
    return w1, w3, w2


def expert_rank(wl: Workload) -> np.ndarray:
    """Popularity rank (1 = hottest) of every expert: a seeded permutation of 1..E, so
    that the local slice holds a mix of hot and cold experts."""
    return _rng(wl, "rank").permutation(wl.E).astype(np.int64) + 1


def skew_roles(wl: Workload):
    """For the skew workload: (hot local experts, never-chosen local experts, cold local experts)."""
    loc = np.arange(wl.e_lo, wl.e_lo + wl.e_cnt)
    hot = loc[[1, wl.e_cnt // 2]] if wl.e_cnt >= 6 else loc[:1]
    n_empty = 3 if wl.e_cnt >= 6 else 1
    empty = loc[[0, wl.e_cnt // 3, wl.e_cnt - 1]][:n_empty] if wl.e_cnt >= 6 else loc[-1:]
    cold = np.array([e for e in loc if e not in set(hot) | set(empty)])
    return hot, empty, cold


def router_weights(wl: Workload) -> np.ndarray:
    """Wr [d,E] ~ N(0,1/d) (second argument = variance), rounded like the workload's dtype: the
    trainable gate's weight matrix."""
    return round_like(wl, _normal(wl, "router", (wl.d, wl.E), wl.d ** -0.5))


def router_logits(wl: Workload, x: np.ndarray | None = None) -> np.ndarray:
    """logits [T,E] fp32 (never bf16-rounded: the router output is fp32).

    router_gemm : x . Wr with Wr ~ N(0,1/d), evaluated here on the host in fp32.
    bias_normal : N(0,1) + per-expert bias ~ N(0, std=bias_std)          (mild imbalance)
    zipf        : N(0,1) - s*ln(rank_e)                                   (Zipf popularity)
    skew        : routing by construction -- half of the local slots land on two hot
                  experts, three local experts are never chosen; selected experts get
                  logit +4+U(0,1), all others -4+U(0,1).
    """
    T, E = wl.T, wl.E
    if wl.routing == "router_gemm":
        if x is None:
            x = tokens(wl)
        wr = _normal(wl, "router", (wl.d, E), wl.d ** -0.5)
        return np.ascontiguousarray((x.astype(np.float32) @ wr).astype(np.float32))
    noise = _normal(wl, "router", (T, E), 1.0)
    if wl.routing == "bias_normal":
        bias = _normal(wl, "bias", (E,), wl.bias_std)
        return noise + bias[None, :]
    if wl.routing == "zipf":
        bias = (-wl.zipf_s * np.log(expert_rank(wl).astype(np.float64))).astype(np.float32)
        return noise + bias[None, :]
    if wl.routing == "skew":
        return _skew_logits(wl)
    raise ValueError(wl.routing)


def _skew_logits(wl: Workload) -> np.ndarray:
    T, E, k = wl.T, wl.E, wl.k
    g = _rng(wl, "route")
    hot, empty, cold = skew_roles(wl)
    # expected local slots per token = 1 (the GPU's fair share k*e_cnt/E at the headline shape)
    share = k * wl.e_cnt / E
    p_hot = 0.5 * share / len(hot)
    p_cold = 0.5 * share / max(len(cold), 1)
    sel = np.zeros((T, E), dtype=bool)
    sel[:, hot] = g.random((T, len(hot))) < p_hot
    if len(cold):
        sel[:, cold] = g.random((T, len(cold))) < p_cold
    nonlocal_ids = np.array([e for e in range(E) if not (wl.e_lo <= e < wl.e_lo + wl.e_cnt)])
    # rank all experts per token by a random score; chosen locals first, then random
    # non-local fill; local experts that were not chosen can never be picked.
    score = g.random((T, E))
    score[sel] += 2.0
    if len(nonlocal_ids):
        score[:, nonlocal_ids] += 1.0
    else:                       # all experts local: fill from the cold ones
        score[:, cold] += 1.0
        score[sel] += 1.0
    score[:, empty] = -1.0
    order = np.argsort(-score, axis=1, kind="stable")[:, :k]
    chosen = np.zeros((T, E), dtype=bool)
    np.put_along_axis(chosen, order, True, axis=1)
    u = g.random((T, E), dtype=np.float32)
    return np.where(chosen, np.float32(4.0) + u, np.float32(-4.0) + u).astype(np.float32)
