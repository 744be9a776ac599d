"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding and
compare each artefact with the CPU oracle on the same seeded inputs."""
import numpy as np
import torch

from oracle import moe_oracle as O
from paper_2605_11005_amd import workloads as W
from paper_2605_11005_amd.layer import MoeLayerBuffers, run_backward, run_forward, upload

# spec tolerances: max |gpu - oracle| / max |oracle| per tensor
TOL = {"f32": 1e-5, "bf16": 2e-2}


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64) if t.is_floating_point() else t.cpu().numpy()


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    scale = np.abs(ref).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / scale)


def elementwise_err(got, ref):
    """Element-wise relative error with an absolute floor of 1e-3 * max|ref| in the denominator:
    returns (largest value, fraction of elements above the bf16 tolerance).  Reported beside the
    max-norm figure: it shows errors confined to small-magnitude elements, which the max-norm hides.
    (No pass/fail bound is attached: after one bf16 rounding of an O(1) intermediate the absolute
    error of every element is a few 1e-3 of the tensor's scale, so elements near the floor sit at O(1).)"""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0
    floor = 1e-3 * np.abs(ref).max()
    if floor == 0.0:
        return float(np.abs(got).max()), float((got != 0).mean())
    e = np.abs(got - ref) / np.maximum(np.abs(ref), floor)
    return float(e.max()), float((e > TOL["bf16"]).mean())


def rms_err(got, ref):
    """||got - ref||_2 / ||ref||_2: a wrong or missing block of any magnitude moves it."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    n = np.sqrt((ref * ref).sum())
    if n == 0.0:
        return float(np.sqrt(((got - ref) ** 2).sum()))
    return float(np.sqrt(((got - ref) ** 2).sum()) / n)


def make_inputs(wl):
    x = W.tokens(wl)
    logits = W.router_logits(wl, x)
    dy = W.out_grad(wl)
    w1, w3, w2 = W.all_expert_weights(wl)
    return dict(x=x, logits=logits, dy=dy, w1=w1, w3=w3, w2=w2)


def oracle_layer(wl, inp):
    fw = O.layer_fwd(inp["x"], inp["logits"], wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt, inp["w1"], inp["w3"], inp["w2"])
    bw = O.layer_bwd(fw, inp["dy"], wl.k, inp["w1"], inp["w3"], inp["w2"])
    return fw, bw


def gpu_layer(wl, inp, cap=None, accumulate=False, poison=True):
    dev = upload(wl, inp["x"], inp["logits"], inp["dy"], inp["w1"], inp["w3"], inp["w2"])
    cap = wl.T * min(wl.k, wl.e_cnt) if cap is None else cap
    buf = MoeLayerBuffers(wl, cap=max(cap, 1))
    if poison:      # outputs must not depend on what the buffers held before; NaN shows an unwritten element
        for name in ("xp", "h1", "h3", "o", "y", "d_o", "dxp", "dx"):
            getattr(buf, name).fill_(float("nan"))
        if not accumulate:
            for name in ("dw1", "dw3", "dw2"):
                getattr(buf, name).fill_(float("nan"))
    run_forward(wl, dev, buf)
    run_backward(wl, dev, buf, accumulate=accumulate)
    torch.cuda.synchronize()
    return dev, buf


def check_layer(wl, inp, fw, bw, buf, tol=None):
    """Integer artefacts bit-exact, floating point within tol.  Returns {name: error}."""
    tol = TOL[wl.dtype] if tol is None else tol
    R = int(fw["offsets"][-1])
    assert buf.status() == 0
    assert (host(buf.topk_idx) == fw["topk_idx"]).all(), "topk_idx"
    assert (host(buf.counts) == fw["counts"]).all(), "counts"
    assert (host(buf.offsets) == fw["offsets"]).all(), "offsets"
    assert (host(buf.perm)[:R] == fw["perm"]).all(), "perm"
    assert (host(buf.inv) == fw["inv"]).all(), "inv"
    # every element the calls own has been written (the buffers were filled with NaN beforehand)
    for name in ("xp", "h1", "h3", "o", "d_o", "dxp"):
        assert torch.isfinite(getattr(buf, name)[:R]).all().item(), f"{name}: unwritten or non-finite element in rows < R"
    for name in ("y", "dx", "dw1", "dw3", "dw2"):
        assert torch.isfinite(getattr(buf, name)).all().item(), f"{name}: unwritten or non-finite element"
    errs = {}
    errs["topk_w"] = float(np.abs(host(buf.topk_w) - fw["topk_w"]).max())
    assert errs["topk_w"] < 1e-5
    # the un-scaled dispatch is a copy: exact
    assert (host(buf.xp)[:R] == fw["xp"]).all(), "xp"
    pairs = [("h1", buf.h1[:R], fw["h1"]), ("h3", buf.h3[:R], fw["h3"]), ("o", buf.o[:R], fw["o"]),
             ("y", buf.y, fw["y"]), ("d_o", buf.d_o[:R], bw["d_o"]), ("dxp", buf.dxp[:R], bw["dxp"]),
             ("dx", buf.dx, bw["dx"])]
    rms = {}
    for name, got, ref in pairs:
        g = host(got)
        errs[name] = rel_err(g, ref)
        rms[name] = rms_err(g, ref)
    for name, got, ref in (("dw1", buf.dw1, bw["dw1"]), ("dw3", buf.dw3, bw["dw3"]), ("dw2", buf.dw2, bw["dw2"])):
        g = host(got)
        worst = 0.0
        for e in range(wl.e_cnt):
            if fw["counts"][e] == 0:
                assert not g[e].any(), f"{name}[{e}] of an empty expert must be zero"
            else:
                worst = max(worst, rel_err(g[e], ref[e]))
                rms[name] = max(rms.get(name, 0.0), rms_err(g[e], ref[e]))
        errs[name] = worst
    bad = {k: v for k, v in errs.items() if not v < tol}
    assert not bad, f"{wl.name}: over tolerance {tol}: {bad} (all: {errs})"
    bad = {k: v for k, v in rms.items() if not v < tol}
    assert not bad, f"{wl.name}: relative l2 error over tolerance {tol}: {bad}"
    return errs
