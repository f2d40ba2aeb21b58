#!/usr/bin/env python3
"""Benchmark of the 1D dilated convolution hot path on one MI355X.

A "step" is one forward + one backward-data + one backward-weight pass of the layer on the
genomics-shaped workload (N=16, C=K=15, W=60000, S=51, d=8, same padding), inputs resident in
HBM.  Prints ONE JSON line:  metric/value = TFLOP/s over the whole step (3 passes x 2*N*C*K*S*Q
nominal FLOPs), plus per-pass figures, a roofline object for the kernel with the largest share of the step
(timed with HIP events on the launch stream) and the FP64 oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"bf16": 2500.0, "fp32": 157.3}      # dense MFMA TFLOP/s, MI355X
HBM_PEAK_GBS = 8000.0
PASSES = ("fwd", "bwd_data", "bwd_weight")
REGIONS = 5                                  # timed regions of --steps steps each; the median region is reported


def algorithmic_bytes(wl, p):
    """Bytes one launch must move: read each input once, write each fp32 output once."""
    e = 2 if wl.dtype == "bf16" else 4
    x, dy, w = wl.N * wl.C * wl.W, wl.N * wl.K * wl.Q, wl.K * wl.C * wl.S
    if p == "fwd":
        return x * e + w * e + dy * 4
    if p == "bwd_data":
        return dy * e + w * e + x * 4
    return x * e + dy * e + w * 4


def stored_traffic(workload, pass_name):
    """HBM bytes per launch of one pass, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by a
    plain copy of known size; read from profiles/hbm_traffic.json when that summary exists, else None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)[workload][pass_name]["bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def sweep_table(args, np, torch, binding, inputs) -> int:
    """Median device time (HIP events), TFLOP/s and fraction of the dense MFMA peak per pass and sweep point."""
    if args.sweep == "q":
        # the paper's own grid (Section 4.3): batch 56, output widths 1000 ... 60000, three filter widths per family
        wls = [inputs.q_sweep_point(f, Q, S) for f in inputs.Q_SWEEP_FAMILIES for S in (5, 21, 51) for Q in inputs.Q_SWEEP_Q]
    else:
        wls = list(inputs.sweep(args.sweep)) + ([inputs.WIDE_BF16] if args.sweep == "bf16" else [])
    print(f"# {'workload':26s} " + " ".join(f"| {p:>10s}: kernel family, us, TFLOP/s, % of peak" for p in PASSES))
    for wl in wls:
        dev = {}
        if args.sweep == "q":
            # timing only: U[-1,1] tensors drawn on the device (seeded), the host generator would dominate the run
            gen = torch.Generator(device="cuda").manual_seed(wl.seed)
            tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
            for k, shape in (("x", (wl.N, wl.C, wl.W)), ("w", (wl.K, wl.C, wl.S)), ("dy", (wl.N, wl.K, wl.Q))):
                dev[k] = (torch.rand(shape, generator=gen, device="cuda") * 2 - 1).to(tdt)
        else:
            data = inputs.make_inputs(wl)
            for k in ("x", "w", "dy"):
                if wl.dtype == "bf16":
                    dev[k] = torch.from_numpy(data[k + "_bits"].view(np.int16)).cuda().view(torch.bfloat16)
                else:
                    dev[k] = torch.from_numpy(data[k]).cuda()
        code = 1 if wl.dtype == "bf16" else 0
        y = torch.empty((wl.N, wl.K, wl.Q), dtype=torch.float32, device="cuda")
        dx = torch.empty((wl.N, wl.C, wl.W), dtype=torch.float32, device="cuda")
        dw = torch.empty((wl.K, wl.C, wl.S), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(256, binding.conv1d_bwd_weight_workspace_bytes(*wl.geometry(), code)), dtype=torch.uint8,
                         device="cuda")
        launch = {
            "fwd": lambda: binding.conv1d_fwd(dev["x"], dev["w"], wl.d, wl.P, out=y),
            "bwd_data": lambda: binding.conv1d_bwd_data(dev["dy"], dev["w"], wl.W, wl.d, wl.P, out=dx),
            "bwd_weight": lambda: binding.conv1d_bwd_weight(dev["x"], dev["dy"], wl.S, wl.d, wl.P, out=dw, workspace=ws),
        }
        cols = []
        for i, p in enumerate(PASSES):
            # untimed launches until the clocks have ramped (about 0.1 s of continuous work), then the warm-up
            t_ramp = time.perf_counter()
            while time.perf_counter() - t_ramp < 0.1:
                for _ in range(10):
                    launch[p]()
                torch.cuda.synchronize()
            for _ in range(args.warmup):
                launch[p]()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            torch.cuda.synchronize()
            for a, b in evs:
                a.record()
                launch[p]()
                b.record()
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in evs)[len(evs) // 2]
            tf = wl.flops / (ms * 1e-3) / 1e12
            fam = binding.conv1d_kernel_name(i, *wl.geometry(), code).split("_")[0]
            cols.append(f"| {fam:>7s} {ms * 1e3:8.1f} us {tf:7.1f} TF {100 * tf / PEAK[wl.dtype]:5.1f} %")
        print(f"{wl.name:28s} " + " ".join(cols), flush=True)
    return 0


def protocol_table(args, torch, inputs) -> int:
    """The paper's own measurement (Section 4.3): wall time of net.forward(x) and of out.sum().backward() on a single
    layer, averaged over 20 iterations, framework overhead included (the sum, the all-ones upstream gradient, the
    accumulation into .grad, dtype casts).  Efficiency = nominal FLOPs / time / dense MFMA peak of the input type."""
    import time as _t

    from paper_2104_08002_amd import autograd

    wls = [inputs.GENOMICS_FP32, inputs.GENOMICS_BF16] + [inputs.q_sweep_point(f, Q, 51) for f, Q in (
        ("c15_d8_fp32", 60000), ("c64_d1_fp32", 10000), ("c64_d1_fp32", 60000), ("c32_d4_bf16", 60000), ("c16_d4_bf16", 60000))]
    iters = 20
    print(f"# {'layer':28s} | forward ms, TFLOP/s, % of peak | sum().backward() ms, TFLOP/s (2 passes), % of peak")
    for wl in wls:
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        gen = torch.Generator(device="cuda").manual_seed(wl.seed)
        net = autograd.Conv1d(wl.C, wl.K, wl.S, dilation=wl.d, padding=wl.P, dtype=tdt)
        x = (torch.rand((wl.N, wl.C, wl.W), generator=gen, device="cuda") * 2 - 1).to(tdt).requires_grad_(True)
        tf = tb = 0.0
        for it in range(iters + 3):
            torch.cuda.synchronize()
            t0 = _t.perf_counter()
            out = net.forward(x)
            torch.cuda.synchronize()
            t1 = _t.perf_counter()
            out.sum().backward()
            torch.cuda.synchronize()
            t2 = _t.perf_counter()
            if it >= 3:
                tf += t1 - t0
                tb += t2 - t1
            x.grad = None
            net.weight.grad = None
        tf, tb = tf / iters, tb / iters
        ff, fb = wl.flops / tf / 1e12, 2 * wl.flops / tb / 1e12
        print(f"{wl.name:30s} | {tf * 1e3:8.3f} ms {ff:7.1f} TF {100 * ff / PEAK[wl.dtype]:5.1f} % | {tb * 1e3:8.3f} ms {fb:7.1f} TF "
              f"{100 * fb / PEAK[wl.dtype]:5.1f} %", flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="genomics_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--protocol", action="store_true",
                    help="instead of the headline line: the paper's measurement protocol (Section 4.3) on single layers: "
                         "wall time of net.forward(x) and out.sum().backward() through the autograd wrapper, 20 iterations")
    ap.add_argument("--separate-backward", action="store_true",
                    help="run the backward passes as conv1d_bwd_data + conv1d_bwd_weight instead of one conv1d_bwd call")
    ap.add_argument("--timing", choices=["both", "hot", "cold"], default="both",
                    help="profiling runs: launch only the hot (one buffer set) or only the cold (rotating sets) configuration, "
                         "so that a kernel trace of the run averages one of them")
    ap.add_argument("--no-ubench", action="store_true", help="skip the MFMA-only / copy microbenchmarks (measured peaks)")
    ap.add_argument("--variant", type=int, default=0, help="force a kernel family (0 = auto)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 256 MiB device-to-device copy 5 times (reference for HBM byte counters)")
    ap.add_argument("--passes", default=",".join(PASSES),
                    help="comma-separated subset of passes to run (profiling runs; the headline needs all three)")
    ap.add_argument("--sweep", choices=["fp32", "bf16", "q"],
                    help="instead of the headline line: per-pass device times of the 25 filter-width x dilation "
                         "points (C = K = 64) of that dtype, plus the wide configuration for bf16, one text line each; "
                         "q: the paper's grid of Section 4.3 (batch 56, output widths 1000 ... 60000, four families)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path would shard over the batch axis: forward and backward-data need no communication, "
              "backward-weight one all-reduce of the weight gradient)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2104_08002_amd import binding, build, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 256 << 20, "launches": 5}))
        return 0
    binding.load()
    binding.conv1d_set_variant(args.variant)
    if args.sweep:
        return sweep_table(args, np, torch, binding, inputs)
    if args.protocol:
        return protocol_table(args, torch, inputs)
    wl = inputs.WORKLOADS[args.workload]
    data = inputs.make_inputs(wl)
    code = 1 if wl.dtype == "bf16" else 0
    ws_bytes = max(256, binding.conv1d_bwd_weight_workspace_bytes(*wl.geometry(), code))

    def make_set():
        s = {}
        for k in ("x", "w", "dy"):
            if wl.dtype == "bf16":
                s[k] = torch.from_numpy(data[k + "_bits"].view(np.int16)).cuda().view(torch.bfloat16)
            else:
                s[k] = torch.from_numpy(data[k]).cuda()
        s["y"] = torch.empty((wl.N, wl.K, wl.Q), dtype=torch.float32, device="cuda")
        s["dx"] = torch.empty((wl.N, wl.C, wl.W), dtype=torch.float32, device="cuda")
        s["dw"] = torch.empty((wl.K, wl.C, wl.S), dtype=torch.float32, device="cuda")
        s["ws"] = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        return s

    # Buffer set 0 is the "hot" configuration: the same tensors step after step (for genomics they stay in the 256 MB
    # last-level cache).  The "cold" configuration walks through several sets of distinct tensors with the same
    # contents, so that more than 1 GB passes between two uses of a tensor and every input comes from HBM.
    set_bytes = sum(t.numel() * t.element_size() for t in make_set().values())
    nsets = max(4, -(-(1 << 30) // set_bytes))
    sets = [make_set() for _ in range(nsets)]

    def launch(p, s):
        if p == "fwd":
            binding.conv1d_fwd(s["x"], s["w"], wl.d, wl.P, out=s["y"])
        elif p == "bwd_data":
            binding.conv1d_bwd_data(s["dy"], s["w"], wl.W, wl.d, wl.P, out=s["dx"])
        else:
            binding.conv1d_bwd_weight(s["x"], s["dy"], wl.S, wl.d, wl.P, out=s["dw"], workspace=s["ws"])

    run_passes = tuple(p for p in PASSES if p in args.passes.split(","))

    # A step is forward + both backward passes.  The backward passes go through conv1d_bwd (one call, same results
    # bit for bit) unless --separate-backward asks for conv1d_bwd_data and conv1d_bwd_weight as calls of their own.
    one_call_backward = set(("bwd_data", "bwd_weight")) <= set(run_passes)

    def step_separate(s):
        for p in run_passes:
            launch(p, s)

    def step_one_call(s):
        if "fwd" in run_passes:
            launch("fwd", s)
        binding.conv1d_bwd(s["x"], s["dy"], s["w"], wl.d, wl.P, out_dx=s["dx"], out_dw=s["dw"], workspace=s["ws"])

    step = step_one_call if (one_call_backward and not args.separate_backward) else step_separate

    def timed_regions(cold, step):
        """REGIONS regions of exactly args.steps steps each, every one bracketed by a device synchronisation."""
        out, k = [], 0
        for _ in range(REGIONS):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step(sets[k % nsets] if cold else sets[0])
                k += 1
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0) * 1e3 / args.steps)
        return out

    for i in range(max(args.warmup, 1)):
        step(sets[0])
    for s in sets[1:]:
        step(s)  # every set once: first-touch costs stay out of the cold figure
    # The first ~50 ms of work after an idle period run slower (clocks ramp up): the regions of a cold start showed
    # 96, 88, 84, 82, 80 us per step.  Keep the GPU busy for that long before anything is timed.
    torch.cuda.synchronize()
    t_ramp = time.perf_counter()
    k_ramp = 0
    while time.perf_counter() - t_ramp < 0.1:
        for _ in range(20):
            step(sets[k_ramp % nsets] if args.timing == "cold" else sets[0])  # (a cold-only run stays cold throughout)
            k_ramp += 1
        torch.cuda.synchronize()
    # --timing hot / cold: both figures come from the one configuration asked for (the JSON says so in "timing_mode")
    hot_is_cold, cold_is_hot = args.timing == "cold", args.timing == "hot"
    hot_regions = timed_regions(hot_is_cold, step)
    cold_regions = timed_regions(not cold_is_hot, step)
    separate = None
    if step is step_one_call and args.timing == "both":
        for _ in range(3):
            step_separate(sets[0])
        sep = sorted(timed_regions(False, step_separate))[REGIONS // 2]
        separate = {"ms_per_step": round(sep, 4), "value": round(len(run_passes) * wl.flops / (sep * 1e-3) / 1e12, 3),
                    "what": "the same step with conv1d_bwd_data and conv1d_bwd_weight as two calls"}
    ms_per_step = sorted(hot_regions)[REGIONS // 2]
    ms_per_step_cold = sorted(cold_regions)[REGIONS // 2]
    value = len(run_passes) * wl.flops / (ms_per_step * 1e-3) / 1e12
    value_cold = len(run_passes) * wl.flops / (ms_per_step_cold * 1e-3) / 1e12

    # per-pass device time: HIP events on the stream the kernels are launched on (torch's current stream)
    def event_times(p, cold):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            s = sets[i % nsets] if cold else sets[0]
            a.record()
            if p == "bwd":
                binding.conv1d_bwd(s["x"], s["dy"], s["w"], wl.d, wl.P, out_dx=s["dx"], out_dw=s["dw"], workspace=s["ws"])
            else:
                launch(p, s)
            b.record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in evs)

    per_pass = {}
    for p in run_passes:
        ms = event_times(p, hot_is_cold)
        msc = event_times(p, not cold_is_hot)
        avg, avgc = sum(ms) / len(ms), sum(msc) / len(msc)
        tf = wl.flops / (avg * 1e-3) / 1e12
        gbs = algorithmic_bytes(wl, p) / (avg * 1e-3) / 1e9
        per_pass[p] = {
            "kernel": binding.conv1d_kernel_name(PASSES.index(p), *wl.geometry(), code),
            "avg_us": round(avg * 1e3, 2), "median_us": round(ms[len(ms) // 2] * 1e3, 2),
            "cold_us": round(avgc * 1e3, 2), "cold_median_us": round(msc[len(msc) // 2] * 1e3, 2),
            "tflops": round(tf, 2), "frac_mfma_peak": round(tf / PEAK[wl.dtype], 4),
            "algorithmic_GBps": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "cold_tflops": round(wl.flops / (avgc * 1e-3) / 1e12, 2),
            "cold_algorithmic_GBps": round(algorithmic_bytes(wl, p) / (avgc * 1e-3) / 1e9, 1),
        }
    # Fused epilogues (Section 3's bias, Section 4.4's ReLU and bfloat16 storage): not part of `value`, whose outputs
    # are float; shown because bfloat16 storage halves the dominant HBM term of the forward and backward-data passes.
    epilogue = None
    if wl.dtype == "bf16" and set(("fwd", "bwd_data")) <= set(run_passes) and args.timing == "both":
        bias = torch.zeros(wl.K, dtype=torch.float32, device="cuda")
        for s in sets:
            s["y16"] = torch.empty((wl.N, wl.K, wl.Q), dtype=torch.bfloat16, device="cuda")
            s["dx16"] = torch.empty((wl.N, wl.C, wl.W), dtype=torch.bfloat16, device="cuda")
        rows = {
            "fwd_bias_relu_bf16out": lambda s: binding.conv1d_fwd_ex(s["x"], s["w"], wl.d, wl.P, bias=bias, relu=True,
                                                                      out_bf16=True, out=s["y16"]),
            "bwd_data_bf16out": lambda s: binding.conv1d_bwd_data_ex(s["dy"], s["w"], wl.W, wl.d, wl.P, out_bf16=True,
                                                                     out=s["dx16"]),
        }
        epilogue = {}
        for name, fn in rows.items():
            res = {}
            for cold in (False, True):
                evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
                fn(sets[0])
                torch.cuda.synchronize()
                for i, (a, b) in enumerate(evs):
                    a.record()
                    fn(sets[i % nsets] if cold else sets[0])
                    b.record()
                torch.cuda.synchronize()
                res["cold_us" if cold else "avg_us"] = round(1e3 * sum(a.elapsed_time(b) for a, b in evs) / len(evs), 2)
            nbytes = algorithmic_bytes(wl, name.split("_bias")[0].split("_bf16out")[0]) - 2 * (wl.N * wl.K * wl.Q if name.startswith("fwd") else wl.N * wl.C * wl.W)
            res.update({"algorithmic_bytes": nbytes, "tflops": round(wl.flops / (res["avg_us"] * 1e-6) / 1e12, 2),
                        "frac_mfma_peak": round(wl.flops / (res["avg_us"] * 1e-6) / 1e12 / PEAK[wl.dtype], 4),
                        "algorithmic_GBps": round(nbytes / (res["avg_us"] * 1e-6) / 1e9, 1)})
            epilogue[name] = res
    bwd_one_call = None
    if one_call_backward:
        ms, msc = event_times("bwd", hot_is_cold), event_times("bwd", not cold_is_hot)
        bwd_one_call = {"avg_us": round(1e3 * sum(ms) / len(ms), 2), "median_us": round(ms[len(ms) // 2] * 1e3, 2),
                        "cold_us": round(1e3 * sum(msc) / len(msc), 2),
                        "tflops": round(2 * wl.flops / (sum(ms) / len(ms) * 1e-3) / 1e12, 2)}
    # measured denominators: what this GPU sustains on an MFMA-only loop and on a plain copy
    measured = None
    if not args.no_ubench and args.timing == "both":
        from paper_2104_08002_amd import ubench

        measured = ubench.measure()
    # The dominant kernel is the one with the largest share of the step.  fwd and bwd_data are launches of the same
    # kernel (one launch per pass); bwd_weight is its own kernel plus the small second stage.
    share = {}
    for p in run_passes:
        share.setdefault(per_pass[p]["kernel"], []).append(p)
    dom_kernel = max(share, key=lambda k: sum(per_pass[p]["avg_us"] for p in share[k]))
    dom_passes = share[dom_kernel]
    dom = dom_passes[0]
    avg_us = sum(per_pass[p]["avg_us"] for p in dom_passes) / len(dom_passes)
    cold_us = sum(per_pass[p]["cold_us"] for p in dom_passes) / len(dom_passes)
    alg_bytes = sum(algorithmic_bytes(wl, p) for p in dom_passes) / len(dom_passes)
    # which roof bounds the dominant kernel: time at MFMA peak vs time at HBM peak for its algorithmic work
    t_mfma = wl.flops / (PEAK[wl.dtype] * 1e12)
    t_hbm = alg_bytes / (HBM_PEAK_GBS * 1e9)
    if t_hbm > t_mfma:
        ach, achc = alg_bytes / (avg_us * 1e-6) / 1e9, alg_bytes / (cold_us * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "achieved_cold": round(achc, 1), "frac_cold": round(achc / HBM_PEAK_GBS, 4)}
        if measured:
            roof["measured_peak"] = measured["hbm_copy_gbps"]
            roof["frac_of_measured_peak"] = round(ach / measured["hbm_copy_gbps"], 4)
            roof["frac_cold_of_measured_peak"] = round(achc / measured["hbm_copy_gbps"], 4)
    else:
        ach, achc = wl.flops / (avg_us * 1e-6) / 1e12, wl.flops / (cold_us * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK[wl.dtype], "unit": "TFLOP/s", "frac": round(ach / PEAK[wl.dtype], 4),
                "achieved_cold": round(achc, 2), "frac_cold": round(achc / PEAK[wl.dtype], 4)}
        if measured:
            mp = measured["mfma_bf16_tflops" if wl.dtype == "bf16" else "mfma_fp32_tflops"]
            roof["measured_peak"] = mp
            roof["frac_of_measured_peak"] = round(ach / mp, 4)
            roof["frac_cold_of_measured_peak"] = round(achc / mp, 4)
    roof.update({"kernel": dom_kernel, "passes": dom_passes, "launches_per_step": len(dom_passes), "avg_us": round(avg_us, 2),
                 "cold_us": round(cold_us, 2), "algorithmic_bytes": int(alg_bytes), "traffic": stored_traffic(wl.name, dom)})

    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        oracle.build()
        x64, w64, dy64 = (data[k].astype(np.float64) for k in ("x", "w", "dy"))
        tt = {}
        t = time.perf_counter(); oracle.fwd(x64, w64, wl.d, wl.P); tt["fwd"] = time.perf_counter() - t
        t = time.perf_counter(); oracle.bwd_data(dy64, w64, wl.W, wl.d, wl.P); tt["bwd_data"] = time.perf_counter() - t
        t = time.perf_counter(); oracle.bwd_weight(x64, dy64, wl.S, wl.d, wl.P); tt["bwd_weight"] = time.perf_counter() - t
        tot = sum(tt.values())
        cpu = {"value": round(3 * wl.flops / tot / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"the whole {wl.name} workload once (N={wl.N}), fp64 direct summation, one run per pass: "
                         + ", ".join(f"{k} {v:.2f}s" for k, v in tt.items())}

    out = {
        "metric": "TFLOP/s per step (fwd + bwd_data + bwd_weight), 1 MI355X", "value": round(value, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "backward": "conv1d_bwd (one call for both backward passes)" if step is step_one_call else "conv1d_bwd_data + conv1d_bwd_weight",
        "separate_backward_calls": separate, "bwd_one_call": bwd_one_call,
        "timing_mode": args.timing,
        "timing": f"median of {REGIONS} regions of {args.steps} steps, each between two device synchronisations",
        "regions_ms_per_step": [round(v, 4) for v in hot_regions],
        "cold": {"ms_per_step": round(ms_per_step_cold, 4), "value": round(value_cold, 3),
                 "frac_mfma_peak": round(value_cold / PEAK[wl.dtype], 4),
                 "regions_ms_per_step": [round(v, 4) for v in cold_regions], "buffer_sets": nsets,
                 "bytes_per_set": set_bytes,
                 "what": "the same step walking through distinct buffer sets, so that no tensor is still cached when it is used again"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "C": wl.C, "K": wl.K, "W": wl.W, "S": wl.S, "dilation": wl.d,
                   "padding": wl.P, "Q": wl.Q, "gflop_per_pass": round(wl.flops / 1e9, 3), "outputs": "fp32"},
        "frac_mfma_peak": round(value / PEAK[wl.dtype], 4),
        "passes": list(run_passes), "per_pass": per_pass, "roofline": roof, "cpu_baseline": cpu,
        "epilogue": epilogue, "measured_peak": measured, "library_sources": build.built_hash(),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
