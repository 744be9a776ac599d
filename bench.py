#!/usr/bin/env python3
"""Benchmark of the MoE expert-layer hot path on one MI355X.

A step = route -> dispatch -> expert forward -> combine -> (backward) scaled dispatch of dY
-> expert backward -> combine of dXp, all through the C ABI, inputs resident in HBM.
Prints ONE JSON line: whole-step expert-layer fwd+bwd TFLOP/s (18*R*d*f useful FLOP per
step, R = realised routed rows), the roofline entry of the dominant grouped-GEMM kernel
(timed live with HIP events inside the library), HBM figures for dispatch/combine, and the
CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
FP32_VECTOR_PEAK_TFLOPS = 157.3
HBM_PEAK_GBPS = 8000.0
INFINITY_CACHE_BYTES = 256 << 20

# useful FLOP per routed row, in units of d*f, of each grouped-GEMM kernel
# units of R*d*f FLOP per launch; the backward runs GEMMs that do not depend on each other as one launch
GEMM_FLOP_UNITS = dict(up=4, down=2, da=2, dx=4, wg=2, wgd=4, da_wg=4, dx_wgd=8)
GEMM_KERNEL_NAMES = dict(da_wg="gg_pair<DA,WG>", dx_wgd="gg_pair<DX,WGD>")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="dsv3-like-share")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-router", action="store_true", help="skip the trainable-gate kernels (timed after the step)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--chunks", type=int, nargs="*", default=[],
                    help="also time the token-chunked two-stream schedule with these chunk counts (reported beside "
                         "the headline value, not inside it)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the compact records of the other configurations (default run of the headline workload only)")
    ap.add_argument("--other-steps", type=int, default=5, help="timed steps per workload of the other_workloads block")
    ap.add_argument("--drop-experts-below", type=int, default=0,
                    help="diagnostic: local experts that would receive fewer rows than this are masked out of the routing "
                         "(their logits are set to -1e30, so their tokens go elsewhere and they get no rows); shows what the "
                         "experts with a handful of rows cost.  Not the headline workload: the line says so in config")
    ap.add_argument("--operand-data", choices=["workload", "constant", "zero"], default="workload",
                    help="diagnostic: overwrite tokens, output gradient and expert weights with one constant (or zero) after "
                         "routing; same kernels, same cycles, less switching activity in the matrix cores -- shows how far the "
                         "package power limit, not the instruction stream, sets the rate.  Not the headline workload")
    ap.add_argument("--power-seconds", type=float, default=0.0,
                    help="after the timed region keep running steps for this many seconds while a child process reads the "
                         "package power and shader clock (rocm-smi) once a second; the samples go into `power_and_clock`")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the MFMA-only / copy / vendor-GEMM ceiling kernels (counter runs that only need the step)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, run three plain 1 GiB device copies (a kernel of known HBM "
                         "traffic) so that a rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the expert layer; --gpus must be 1 "
              "(no collectives or multi-GPU sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_11005_amd import binding as B
    from paper_2605_11005_amd import workloads as W

    wl = W.BY_NAME[args.workload]
    B.load_library()
    torch.cuda.set_device(0)
    out, host_inputs = run_workload(wl, args.steps, args.warmup, full=True, args=args)

    if not args.no_other_workloads and args.workload == "dsv3-like-share":
        # The remaining headline configurations and the paper's model-table shapes, after the headline's
        # timed region: whole-step rate, step time and the slowest grouped-GEMM kernel of each.
        others = {}
        for w in [W.MIXTRAL, W.QWEN, W.SKEW] + W.MODEL_TABLE:
            r, _ = run_workload(w, args.other_steps, 2, full=False, args=args)
            others[w.name] = r
        out["other_workloads"] = others

    if not args.no_cpu_baseline:
        x, logits, dy = host_inputs
        out["cpu_baseline"] = cpu_baseline(wl, x, logits, dy, args.cpu_seconds)
    print(json.dumps(out))


def run_workload(wl, steps, warmup, full, args):
    """K timed steps of the whole hot path on one workload.  full=True: the complete record of the
    headline line; full=False: the compact record of the `other_workloads` block."""
    import numpy as np
    import torch
    from paper_2605_11005_amd import binding as B
    from paper_2605_11005_amd import counters as C
    from paper_2605_11005_amd import workloads as W
    from paper_2605_11005_amd.layer import MoeLayerBuffers, run_backward, run_forward, to_device, torch_dtype

    bf16 = wl.dtype == "bf16"
    b = 2 if bf16 else 4
    t0 = time.time()
    x = W.tokens(wl)
    logits = W.router_logits(wl, x)
    dropped = []
    if full and args.drop_experts_below > 0:
        lt = torch.from_numpy(logits).cuda()
        c0 = torch.empty((wl.e_cnt,), dtype=torch.int32, device="cuda")
        B.moe_route(lt, wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt, torch.empty((wl.T, wl.k), dtype=torch.int32, device="cuda"),
                    torch.empty((wl.T, wl.k), dtype=torch.float32, device="cuda"), c0)
        dropped = [wl.e_lo + e for e, c in enumerate(c0.cpu().tolist()) if c < args.drop_experts_below]
        logits = logits.copy()
        logits[:, dropped] = -1e30
        del lt, c0
    dy = W.out_grad(wl)
    w1, w3, w2 = W.all_expert_weights(wl, out_bits=bf16)
    dt = torch_dtype(wl)
    dev = dict(x=to_device(x, dt), logits=to_device(logits, torch.float32), dy=to_device(dy, dt),
               w1=to_device(w1, dt, bf16), w3=to_device(w3, dt, bf16), w2=to_device(w2, dt, bf16))
    del w1, w3, w2
    if full and args.operand_data != "workload":
        for name, val in (("x", 1.0), ("dy", 1.0), ("w1", 0.5), ("w3", 0.5), ("w2", 0.5)):
            dev[name].fill_(val if args.operand_data == "constant" else 0.0)
    gen_s = time.time() - t0

    # realised row count (outside the timed region) sizes the expert-order buffers
    cnt = torch.empty((wl.e_cnt,), dtype=torch.int32, device="cuda")
    ti = torch.empty((wl.T, wl.k), dtype=torch.int32, device="cuda")
    tw = torch.empty((wl.T, wl.k), dtype=torch.float32, device="cuda")
    B.moe_route(dev["logits"], wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt, ti, tw, cnt)
    counts = cnt.cpu().numpy()
    R = int(counts.sum())
    local = ((ti >= wl.e_lo) & (ti < wl.e_lo + wl.e_cnt))
    U = int(local.any(dim=1).sum().item())
    del ti, tw, cnt, local
    cap = max(R, 1)
    buf = MoeLayerBuffers(wl, cap=cap)

    def step():
        run_forward(wl, dev, buf)
        run_backward(wl, dev, buf)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    assert buf.status() == 0

    # ---- timed region: exactly K steps, kernels bracketed by events inside the library
    B.moe_profile_enable(True)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t_start = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step()
        marks[i + 1].record()     # asynchronous: per-step times for the min / median beside the bracketed mean
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    B.moe_profile_enable(False)
    ms_per_step = elapsed * 1e3 / steps

    kern = {}
    for name in B.KERNEL_IDS:
        ms, n = B.moe_profile_read(name)
        if n:
            lo, med = B.moe_profile_stats(name)
            kern[name] = dict(avg_ms=ms / n, min_ms=lo, median_ms=med, launches=n)

    d, f, T, k = wl.d, wl.f, wl.T, wl.k
    flop_step = C.layer_flops(R, d, f)
    value = flop_step / (ms_per_step * 1e-3) / 1e12
    # per step: the grouped-GEMM launches (six GEMMs in four launches: dA with dW2, dX with dW1|dW3) plus the two
    # partial-tile reductions of cut weight gradients
    gemm_ms = sum(kern[n]["avg_ms"] * kern[n]["launches"] for n in list(GEMM_FLOP_UNITS) + ["wgrad_reduce"] if n in kern) / steps
    for name, units in GEMM_FLOP_UNITS.items():
        if name in kern:
            kern[name]["tflops"] = C.gemm_flops(R, d, f, units / 2) / (kern[name]["avg_ms"] * 1e-3) / 1e12
    # algorithmic bytes of the row movers: dispatch (U+R) rows + index traffic, combine (R+T) rows
    disp_bytes = C.dispatch_bytes(U, R, T, k, d, b)
    comb_bytes = C.combine_bytes(R, T, k, d, b)
    if "dispatch" in kern:
        kern["dispatch"]["GBps"] = disp_bytes / (kern["dispatch"]["avg_ms"] * 1e-3) / 1e9
    if "combine" in kern:
        kern["combine"]["GBps"] = comb_bytes / (kern["combine"]["avg_ms"] * 1e-3) / 1e9

    roofline = None
    if bf16:
        dom = max((n for n in GEMM_FLOP_UNITS if n in kern), key=lambda n: kern[n]["avg_ms"])
        kname = GEMM_KERNEL_NAMES.get(dom, f"gg_kernel<{dom.upper()}>")
        roofline = dict(kernel=kname, bound="mfma", achieved=kern[dom]["tflops"],
                        peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s", frac=kern[dom]["tflops"] / MFMA_BF16_PEAK_TFLOPS,
                        traffic=measured_traffic(wl.name, kname),
                        all_gemms_tflops=C.layer_flops(R, d, f) / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None)
        # experts with few rows are bound by reading their weights, not by MFMA: composite bound
        comp_ms = 1e3 * C.expert_composite_bound_s(counts.tolist(), d, f, b, MFMA_BF16_PEAK_TFLOPS * 1e12,
                                                   HBM_PEAK_GBPS * 1e9)
        roofline["composite_bound_ms"] = comp_ms
        roofline["all_gemms_ms"] = gemm_ms
        roofline["all_gemms_frac_of_composite_bound"] = comp_ms / gemm_ms if gemm_ms else None
    else:
        # fp32 path: plain FMA tiles on the vector ALUs
        fl = C.layer_flops(R, d, f)
        roofline = dict(kernel="fp32 expert GEMMs (all)", bound="alu", achieved=fl / (ms_per_step * 1e-3) / 1e12,
                        peak=FP32_VECTOR_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=fl / (ms_per_step * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS, traffic=None)
    # Within a step every mover launch touches other data than the one before it (x, then o, then dy,
    # then dxp), so a launch re-reads nothing it left in a cache itself; but a launch whose bytes fit the
    # 256 MB Infinity Cache may find its input there, written by the kernel before it: labelled.
    hbm = {}
    for name, nbytes in (("dispatch", disp_bytes), ("combine", comb_bytes)):
        if name in kern:
            hbm[name] = dict(bound="hbm", achieved=kern[name]["GBps"], peak=HBM_PEAK_GBPS, unit="GB/s",
                             frac=kern[name]["GBps"] / HBM_PEAK_GBPS, bytes_per_launch=nbytes,
                             may_fit_infinity_cache=bool(nbytes < INFINITY_CACHE_BYTES))
    config = {"workload": wl.name, "T": T, "d": d, "E": wl.E, "local_experts": wl.e_cnt, "k": k, "f": f,
              "gate_mode": wl.gate_mode, "routed_rows_R": R, "tokens_with_local_slot_U": U,
              "rows_per_expert_min_max": [int(counts.min()), int(counts.max())]}
    if full and args.operand_data != "workload":
        config["workload"] = wl.name + f" with {args.operand_data} operand data (diagnostic)"
    if dropped:
        config["workload"] = wl.name + f" with {len(dropped)} local experts below {args.drop_experts_below} rows masked out of the routing"
        config["experts_masked_out"] = dropped
    if not full:
        rec = {"value": value, "unit": "TFLOP/s", "ms_per_step": ms_per_step, "steps": steps, "dtype": wl.dtype,
               "config": config,
               "dominant_kernel": {"kernel": roofline["kernel"], "achieved": roofline["achieved"], "frac": roofline["frac"]},
               "all_gemms_tflops": roofline.get("all_gemms_tflops"),
               "all_gemms_frac_of_composite_bound": roofline.get("all_gemms_frac_of_composite_bound"),
               "dispatch_combine_GBps": [hbm.get("dispatch", {}).get("achieved"), hbm.get("combine", {}).get("achieved")],
               "dispatch_combine_may_fit_infinity_cache": [hbm.get("dispatch", {}).get("may_fit_infinity_cache"),
                                                           hbm.get("combine", {}).get("may_fit_infinity_cache")]}
        del dev, buf
        torch.cuda.empty_cache()
        return rec, None

    power = power_and_clock(torch, step, args.power_seconds) if args.power_seconds > 0 else None
    # enabling the profiler again starts a new log: the step's figures were read above
    router = None if args.no_router else router_row(B, C, W, torch, wl, dev, buf, R, U, b)
    chunked = {str(c): chunked_ms(torch, wl, dev, c, warmup, steps) for c in args.chunks}
    ceilings = None if args.no_ceilings else measured_ceilings(B, torch)

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "expert-layer fwd+bwd TFLOP/s", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "ms_per_step_min": per_step[0], "ms_per_step_median": per_step[len(per_step) // 2], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": config,
        "roofline": roofline, "hbm_kernels": hbm, "measured_ceilings": ceilings, "kernels": kern,
        "dispatch_combine_GBps": [hbm.get("dispatch", {}).get("achieved"), hbm.get("combine", {}).get("achieved")],
        "input_generation_s": gen_s,
    }
    if power:
        out["power_and_clock"] = power
    if router:
        out["trainable_gate"] = router
    if chunked:
        out["chunked_schedule_ms_per_step"] = chunked
    del dev, buf
    torch.cuda.empty_cache()
    return out, (x, logits, dy)


def power_and_clock(torch, step, seconds):
    """Package power and shader clock while the steps run back to back: a sampler thread starts `rocm-smi` as a
    child process about once a second (a read-only query) while this thread keeps the GPU busy."""
    import re
    import subprocess
    import threading
    samples, stop = [], threading.Event()

    def find(obj, name):
        """First value stored under a key called `name` anywhere in a nested JSON object."""
        if isinstance(obj, dict):
            for key, val in obj.items():
                if key.lower() == name:
                    return val
                got = find(val, name)
                if got is not None:
                    return got
        elif isinstance(obj, list):
            for val in obj:
                got = find(val, name)
                if got is not None:
                    return got
        return None

    def number(val):
        if isinstance(val, dict):
            val = val.get("value")
        m = re.search(r"([0-9]+(?:\.[0-9]+)?)", str(val))
        return float(m.group(1)) if m else None

    def sampler():
        time.sleep(min(3.0, seconds / 4))            # let the clocks settle under load first
        while not stop.is_set():
            rec = {}
            try:                                     # shader clock and the power limit
                txt = subprocess.run(["rocm-smi", "--showclocks", "--showmaxpower", "--json"], capture_output=True, text=True,
                                     timeout=10).stdout
                for key, val in next(iter(json.loads(txt).values())).items():
                    lk = key.lower()
                    if "max" in lk and "power" in lk:
                        rec["power_cap_W"] = number(val)
                    elif lk.startswith("sclk") and "level" not in lk:
                        rec["sclk_MHz"] = number(val)
            except Exception as exc:                 # the queries are a courtesy: report, never fail the benchmark
                rec["rocm_smi_error"] = str(exc)[:200]
            try:                                     # package (socket) power
                txt = subprocess.run(["amd-smi", "metric", "-g", "0", "--power", "--json"], capture_output=True, text=True,
                                     timeout=10).stdout
                val = find(json.loads(txt), "socket_power")
                if val is not None:
                    rec["package_power_W"] = number(val)
            except Exception as exc:
                rec["amd_smi_error"] = str(exc)[:200]
            samples.append(rec)
            stop.wait(1.0)

    th = threading.Thread(target=sampler, daemon=True)
    th.start()
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        n += 5
    busy = time.perf_counter() - t0
    stop.set()
    th.join(timeout=15)
    def med(key):
        vals = sorted(r[key] for r in samples if r.get(key) is not None)
        return vals[len(vals) // 2] if vals else None

    return {"seconds": busy, "steps": n, "ms_per_step": busy * 1e3 / n if n else None, "samples": samples,
            "median_package_power_W": med("package_power_W"), "median_sclk_MHz": med("sclk_MHz"),
            "power_cap_W": med("power_cap_W")}


def router_row(B, C, W, torch, wl, dev, buf, R, U, b, reps=10):
    """The trainable-gate kernels at this workload, timed on their own after the step (they are
    not part of `value`): router GEMM, fused backward of combine, gate backward, router backward."""
    T, d, E, k = wl.T, wl.d, wl.E, wl.k
    dt = dev["x"].dtype
    code = B.MOE_BF16 if wl.dtype == "bf16" else B.MOE_F32
    wr = torch.from_numpy(W.router_weights(wl)).cuda().to(dt)
    logits = torch.empty((T, E), dtype=torch.float32, device="cuda")
    dgate = torch.empty((T, k), dtype=torch.float32, device="cuda")
    dlogits = torch.empty((T, E), dtype=torch.float32, device="cuda")
    dwr = torch.empty((d, E), dtype=dt, device="cuda")
    ws = torch.empty(B.moe_workspace_bytes(B.WS_ROUTER, code, T, k, d, wl.f, E, 0), dtype=torch.uint8, device="cuda")

    def run():
        B.moe_router_fwd(dev["x"], wr, logits, ws)
        B.moe_combine_bwd(dev["dy"], buf.o, buf.inv, buf.topk_w, buf.d_o, dgate)
        B.moe_gate_bwd(dev["logits"], buf.topk_idx, dgate, wl.gate_mode, dlogits)
        B.moe_router_bwd(dev["x"], wr, dlogits, dwr, False, buf.dx, True, ws)

    for _ in range(3):
        run()
    torch.cuda.synchronize()
    B.moe_profile_enable(True)
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    B.moe_profile_enable(False)
    out = {}
    gemm_flop = 2.0 * T * d * E
    for name in ("router_fwd", "combine_bwd", "gate_bwd", "router_dw", "router_dx"):
        ms, n = B.moe_profile_read(name)
        if not n:
            continue
        avg = ms / reps             # per call: a call may consist of several launches (rounding, GEMM, reduction)
        out[name] = dict(avg_ms=avg)
        if name in ("router_fwd", "router_dw", "router_dx"):
            out[name]["tflops"] = gemm_flop / (avg * 1e-3) / 1e12
    if "combine_bwd" in out:       # dy rows of tokens with a local slot + o rows read, d_o rows written
        out["combine_bwd"]["GBps"] = ((U + 2 * R) * d * b + 12.0 * T * k) / (out["combine_bwd"]["avg_ms"] * 1e-3) / 1e9
    if "router_dx" in out:         # dx read and written, dlogits and Wr read
        out["router_dx"]["GBps"] = (2.0 * T * d * b + T * E * 2 + d * E * b) / (out["router_dx"]["avg_ms"] * 1e-3) / 1e9
    out["total_ms"] = sum(v["avg_ms"] for v in out.values())
    return out


def chunked_ms(torch, wl, dev, n_chunks, warmup, steps):
    """Step time of the token-chunked two-stream schedule (movers of one chunk beside the GEMMs of another)."""
    from paper_2605_11005_amd.chunked import ChunkedLayer
    ch = ChunkedLayer(wl, n_chunks)
    for _ in range(max(warmup, 1)):
        ch.forward(dev); ch.backward(dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ch.forward(dev); ch.backward(dev)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def measured_ceilings(B, torch):
    """What this machine sustains, measured in the same run (outside the timed region): MFMA-only bf16
    loops with constant and with pseudo-random operands, and a plain 1 GiB device copy."""
    sink = torch.empty(1024 * 256, dtype=torch.float32, device="cuda")
    out = {}

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    for tag, rnd in (("mfma_bf16_constant_operands_TFLOPs", False), ("mfma_bf16_random_operands_TFLOPs", True)):
        flop = B.moe_probe_mfma_bf16(sink, 4000, rnd)
        t = timed(lambda: B.moe_probe_mfma_bf16(sink, 4000, rnd), 20)    # ~20 ms of sustained load
        out[tag] = flop / t / 1e12
    # the same loop with random operands re-read from LDS at the grouped GEMM's rate: what the matrix cores
    # sustain under the package power limit once their operand feed is paid for
    for tag, feed in (("mfma_bf16_random_operands_lds_16B_reads_TFLOPs", 1), ("mfma_bf16_random_operands_lds_transposing_reads_TFLOPs", 2)):
        flop = B.moe_probe_mfma_fed_bf16(sink, 4000, feed)
        t = timed(lambda: B.moe_probe_mfma_fed_bf16(sink, 4000, feed), 20)
        out[tag] = flop / t / 1e12
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    t = timed(lambda: B.moe_probe_copy(src, dst), 10)
    out["device_copy_GBps"] = 2.0 * (1 << 30) / t / 1e9
    # streaming kernels with the row movers' access width over 1 GiB: fill, read, one read fanned out to two
    # writes (the dispatch's mix at the headline share: 2.2 rows written per row read)
    word = torch.zeros(16, dtype=torch.int32, device="cuda")
    for tag, writes, moved in (("stream_fill_GBps", 0, 1.0), ("stream_read_GBps", -1, 1.0), ("stream_1_read_2_writes_GBps", 2, 3.0)):
        t = timed(lambda: B.moe_probe_stream(src, dst, writes, word), 10)
        out[tag] = moved * (1 << 30) / t / 1e9
    del src, dst
    # yardstick only: the vendor library's dense bf16 GEMM (torch.matmul) on one large problem of
    # the up-projection's shape and operand layout, random operands
    M, K, N = 65536, 7168, 4096
    a = torch.randn((M, K), device="cuda", dtype=torch.bfloat16)
    w = torch.randn((K, N), device="cuda", dtype=torch.bfloat16) * K ** -0.5
    t = timed(lambda: torch.matmul(a, w), 10)
    out["vendor_dense_gemm_bf16_TFLOPs"] = 2.0 * M * N * K / t / 1e12
    return out


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    summary of this workload (a counter run cannot happen inside the benchmark); None if absent."""
    path = os.path.join(ROOT, "profiles", {"dsv3-like-share": "hot_path_dsv3_hbm_traffic.md"}.get(workload, ""))
    if not os.path.isfile(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return json.loads(line.split(":", 1)[1]).get(kernel)
    return None


def cpu_baseline(wl, x, logits, dy, budget_s):
    """The oracle as it stands, on the host cores: route/plan/dispatch/combine at full size,
    the expert forward+backward on as many local experts (in id order) as fit the budget."""
    import numpy as np
    from oracle import moe_oracle as O
    from paper_2605_11005_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        cores = max((p.get("num_threads", 1) for p in threadpool_info()), default=1)
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.perf_counter()
    topk_idx, topk_w, counts = O.route(logits, wl.k, wl.gate_mode, wl.e_lo, wl.e_cnt)
    offsets, perm, inv = O.plan(topk_idx, wl.e_lo, wl.e_cnt)
    xp = O.dispatch(x, perm, wl.k)
    d_o = O.dispatch(dy, perm, wl.k, row_scale=topk_w)
    t_perm = time.perf_counter() - t0
    flops = 0.0
    t_exp = 0.0
    done = []
    rows = 0
    for e in range(wl.e_cnt):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        w1, w3, w2 = W.expert_weights(wl, e)
        off1 = np.array([0, hi - lo], dtype=np.int32)
        t1 = time.perf_counter()
        h1, h3, a, o = O.expert_fwd(xp[lo:hi], off1, [w1], [w3], [w2])
        O.expert_bwd(xp[lo:hi], h1, h3, d_o[lo:hi], off1, [w1], [w3], [w2])
        t_exp += time.perf_counter() - t1
        flops += 18.0 * (hi - lo) * wl.d * wl.f
        rows += hi - lo
        done.append(e)
        if t_exp > budget_s:
            break
    t2 = time.perf_counter()
    O.combine(xp, inv, topk_w)
    t_comb = time.perf_counter() - t2
    return {"value": flops / t_exp / 1e12 if t_exp else None, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"expert fwd+bwd of local experts {done} ({rows} of {int(offsets[-1])} routed rows) in "
                      f"{t_exp:.1f} s; route+plan+2 dispatches at full size in {t_perm:.1f} s, one combine in "
                      f"{t_comb:.1f} s (numpy float64)",
            "expert_seconds": t_exp, "permute_seconds": t_perm + t_comb}


if __name__ == "__main__":
    main()
