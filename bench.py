#!/usr/bin/env python3
"""Benchmark of the depthwise-convolution hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: forward,
input gradient, and weight gradient (stage 1 + stage 2), through the C ABI, at the
headline training-step shape (fp32 B32 C256 L4096 K64 causal) unless --workload says
otherwise.  Inputs are resident in HBM before the timed region; buffers rotate over
several sets so that no step finds what an earlier step left in the 256 MB last-level
cache.  Within a step the weight gradient re-reads x and dY after the forward and
input-gradient launches have read them, as a training step does, and the library keeps
its outputs out of that cache (streaming stores) so that part of them is still there.

Prints ONE JSON line:  metric / value = effective HBM GB/s of the full step (algorithmic
bytes: each path reads two [B,C,L] tensors' worth and one [C,K], i.e. reads two and
writes one), ms_per_step, per-path microseconds, a `roofline` object for the kernel that
dominates the step, and a `cpu_baseline` object (the fp64 CPU oracle timed on host cores).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=1, help="index into workloads.WORKLOADS (1 = headline)")
    ap.add_argument("--shape", nargs=6, metavar=("B", "C", "L", "K", "PAD", "DTYPE"), default=None,
                    help="instead of a listed workload: any shape, e.g. --shape 32 256 4096 256 255 f32 "
                         "(filters N(0, 1/K); no stored traffic figure; combine with --no-cpu-baseline for large K)")
    ap.add_argument("--sets", type=int, default=4, help="rotating buffer sets")
    ap.add_argument("--min-warm-s", type=float, default=1.0,
                    help="keep warming up (whole steps, beyond --warmup) until this much wall time has been spent on "
                         "warm-up steps: a short run must not time the part's clock ramp (0 = exactly --warmup steps)")
    ap.add_argument("--trace-steps", type=int, default=16,
                    help="per-step event times of the first N steps after set-up, reported as first_steps_us "
                         "(they are warm-up steps; nothing is hidden: the ramp shows here)")
    ap.add_argument("--data", choices=("workload", "zeros"), default="workload",
                    help="zeros: all-zero x, w and dY (same work; the part draws less power, so the shader clock the "
                         "kernels sustain on real data can be told from the clock-free time; no parity meaning)")
    ap.add_argument("--sample-clocks", action="store_true",
                    help="sample `rocm-smi --showclocks` while the timed region runs and report the shader clock seen")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-roof", action="store_true",
                    help="instead of the benchmark, time plain device copies of 128 MiB .. 1 GiB (what a streaming "
                         "read + write reaches on this part, with and without help from the last-level cache)")
    return ap.parse_args()


def cpu_baseline(wl, inputs):
    """The oracle as it stands, timed on the host cores: one full step of the same workload
    (or, for workloads whose step exceeds ~30 s of CPU work, a bounded slice of it)."""
    import numpy as np
    import oracle
    from paper_2604_25422_amd.roofline import algorithmic_bytes
    from paper_2604_25422_amd.workloads import as_f32_numpy
    oracle.build()
    # ~3e9 fp64 MAC/s on 8 cores; keep the sample to roughly 10-30 s of CPU work
    Bs, Cs = wl.B, wl.C
    while 3.0 * Bs * Cs * wl.L * min(wl.K, wl.L) > 4.0e10 and Cs > 1:
        Cs = max(1, Cs // 2)
    x = np.ascontiguousarray(as_f32_numpy(inputs["x"])[:Bs, :Cs])
    dy = np.ascontiguousarray(as_f32_numpy(inputs["dy"])[:Bs, :Cs])
    w = np.ascontiguousarray(as_f32_numpy(inputs["w"])[:Cs])
    def one_step():
        t0 = time.perf_counter()
        oracle.fwd(x, w, wl.pad_left)
        oracle.bwd_input(dy, w, wl.pad_left)
        oracle.bwd_weight(x, dy, wl.K, wl.pad_left)
        return time.perf_counter() - t0

    first = one_step()
    # repeat short steps so the sample is about 10-30 s of CPU work (wall time x threads), at most 8 times
    reps = max(1, min(8, int(20.0 / max(first * oracle.threads(), 1e-3))))
    times = [first] + [one_step() for _ in range(reps - 1)]
    dt = sum(times) / len(times)
    nbytes = algorithmic_bytes(Bs, Cs, wl.L, wl.K, wl.elem_size, "step")
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
            "seconds": dt, "repeats": len(times),
            "sample": f"one full fwd+dX+dW step of B{Bs} C{Cs} L{wl.L} K{wl.K} "
                      f"({'the whole workload' if (Bs, Cs) == (wl.B, wl.C) else 'a channel slice of the workload'}), "
                      f"fp64 accumulate, OpenMP over rows/coefficients"}


def measure_copies(sizes_mib):
    """Plain device-to-device copies, 20 back to back after 3 warm-ups: read + write GB/s per size."""
    import torch
    out = {}
    for mib in sizes_mib:
        n = mib * (1 << 20) // 4
        a = torch.ones(n, dtype=torch.float32, device="cuda"); b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize(); e0.record()
        for _ in range(20):
            b.copy_(a)
        e1.record(); torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 20 * 1e3
        out[f"{mib}MiB"] = {"us": round(us, 1), "GBps": round(2 * n * 4 / (us * 1e-6) / 1e9, 1)}
        del a, b
    return out


def copy_roof():
    out = measure_copies((128, 256, 1024))
    print(json.dumps({"copy_roof": out, "note": "same source and destination every repetition: up to 256 MiB the "
                      "source stays in the 256 MB last-level cache, 1 GiB is served by HBM alone"}), flush=True)


def main():
    args = parse_args()
    if args.copy_roof:
        copy_roof()
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists: channels shard "
              "without communication, batches need one all-reduce of dW)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_25422_amd import binding, workloads
    from paper_2604_25422_amd.roofline import (HBM_PEAK_GBPS, MFMA_BF16_PEAK_TFLOPS, MFMA_F32_PEAK_TFLOPS, algorithmic_bytes, dense_flops,
                                               in_range_flops, measured_traffic)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.lib()   # fail loudly if the HIP library is missing
    wl = workloads.WORKLOADS[args.workload]
    if args.shape is not None:
        B_, C_, L_, K_, P_ = (int(v) for v in args.shape[:5])
        dt_ = args.shape[5]
        if dt_ not in ("f32", "bf16") or min(B_, C_, L_, K_) < 1 or not 0 <= P_ < K_:
            print("bench.py: --shape B C L K PAD DTYPE with 0 <= PAD < K and DTYPE f32 or bf16", file=sys.stderr)
            sys.exit(2)
        wl = workloads.Workload(f"shape_B{B_}_C{C_}_L{L_}_K{K_}_pad{P_}_{dt_}", 99, B_, C_, L_, K_, P_, dt_, "normal_var_1_over_K")
        args.workload = -1
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    inputs = workloads.make_inputs(wl)
    if args.data == "zeros":
        inputs = {k: torch.zeros_like(v) for k, v in inputs.items()}
    K, p = wl.K, wl.pad_left

    sets = []
    for i in range(args.sets):
        s = {"x": inputs["x"].to(dev), "w": inputs["w"].to(dev), "dy": inputs["dy"].to(dev)}
        if i:   # distinct contents per set; values do not change the work done
            s["x"] = s["x"].roll(i, dims=2).contiguous()
            s["dy"] = s["dy"].roll(-i, dims=2).contiguous()
        s["y"] = torch.empty_like(s["x"]); s["dx"] = torch.empty_like(s["x"])
        s["dw"] = torch.empty_like(s["w"])
        s["ws"] = binding.new_workspace(s["x"], K, p)
        sets.append(s)
    tdt = workloads.torch_dtype(wl)

    # The weight gradient runs as one kernel when a whole channel is reduced inside one workgroup; otherwise
    # its two stages are launched (and timed) separately.
    code = binding.F32 if wl.dtype == "f32" else binding.BF16
    single = binding.dwconv_bwd_weight_single_pass(wl.B, wl.C, wl.L, K, p, code)

    def step(s, ev=None):
        if ev: ev[0].record()
        binding.dwconv_fwd(s["x"], s["w"], p, out=s["y"])
        if ev: ev[1].record()
        binding.dwconv_bwd_input(s["dy"], s["w"], p, out=s["dx"])
        if ev: ev[2].record()
        if single:
            binding.dwconv_bwd_weight(s["x"], s["dy"], K, p, workspace=s["ws"], out=s["dw"])
            if ev: ev[3].record()
        else:
            binding.dwconv_bwd_weight_partial(s["x"], s["dy"], K, p, workspace=s["ws"])
            if ev: ev[3].record()
            binding.dwconv_bwd_weight_finalize(s["ws"], wl.B, wl.C, wl.L, K, p, tdt, out=s["dw"])
        if ev: ev[4].record()

    fused_on = bool(binding.dwconv_bwd_is_fused(wl.B, wl.C, wl.L, K, p, code))

    def step_fused(s, ev=None):
        if ev: ev[0].record()
        binding.dwconv_fwd(s["x"], s["w"], p, out=s["y"])
        if ev: ev[1].record()
        binding.dwconv_bwd(s["dy"], s["x"], s["w"], p, workspace=s["ws"], out_dx=s["dx"], out_dw=s["dw"])
        if ev: ev[2].record()

    def new_events(n, k):
        return [[torch.cuda.Event(enable_timing=True) for _ in range(k)] for _ in range(n)]

    # One plain device copy of a known size (x -> y of set 0) before anything is timed: under
    # rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate those counters.
    sets[0]["y"].copy_(sets[0]["x"])
    # Set-up, not warm-up: every kernel of the step is launched once on every buffer set, so that code objects are
    # loaded, the library's per-kernel occupancy and LDS-attribute queries are done and every page is touched.
    for s in sets:
        step(s)
        if fused_on:
            step_fused(s)
    torch.cuda.synchronize()

    # Warm-up: the first `trace_steps` steps carry one event pair each (their times are reported as first_steps_us,
    # so a clock ramp after an idle period shows in the line instead of hiding in the mean); then whole steps until
    # both `warmup` steps and `min_warm_s` seconds of warm-up have run.
    n_trace = max(0, args.trace_steps)
    tev = new_events(n_trace, 2)
    t_warm0 = time.perf_counter()
    for i in range(n_trace):
        tev[i][0].record(); step(sets[i % args.sets]); tev[i][1].record()
    torch.cuda.synchronize()
    first_steps_us = [round(1e3 * e[0].elapsed_time(e[1]), 1) for e in tev]
    warm_done = n_trace
    chunk = max(1, min(64, args.warmup if args.warmup > 0 else 16))
    while warm_done < args.warmup or (time.perf_counter() - t_warm0) < args.min_warm_s:
        n = chunk if warm_done >= args.warmup else min(chunk, args.warmup - warm_done)
        for i in range(n):
            step(sets[(warm_done + i) % args.sets])
        torch.cuda.synchronize()
        warm_done += n
    warm_seconds = time.perf_counter() - t_warm0

    # timed region 1: exactly `steps` steps back to back (the headline number)
    clocks = []
    sampler = None
    if args.sample_clocks:
        import re
        import subprocess
        import threading
        stop_sampling = threading.Event()

        def sample():
            while not stop_sampling.is_set():
                try:
                    o = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=5).stdout
                    m = re.search(r"sclk clock level:.*?\((\d+)Mhz\)", o)
                    if m:
                        clocks.append(int(m.group(1)))
                except Exception:
                    pass
                time.sleep(0.02)
        sampler = threading.Thread(target=sample, daemon=True)
        sampler.start()
    start = torch.cuda.Event(enable_timing=True); end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(args.steps):
        step(sets[i % args.sets])
    end.record()
    torch.cuda.synchronize()
    ms_per_step = start.elapsed_time(end) / args.steps
    if sampler:
        stop_sampling.set()
        sampler.join()

    # timed region 2: the same steps with HIP events between the launches, for per-kernel durations
    # (at least 50 of them, so that median and minimum mean something on a short run)
    n_ev = max(args.steps, 50)
    evs = new_events(n_ev, 5)
    torch.cuda.synchronize()
    for i in range(n_ev):
        step(sets[i % args.sets], evs[i])
    torch.cuda.synchronize()
    names = ["fwd", "dx", "dw_partial", "dw_finalize"]
    samples = {n: sorted(1e3 * e[k].elapsed_time(e[k + 1]) for e in evs) for k, n in enumerate(names)}
    if single:
        samples["dw_finalize"] = [0.0] * n_ev          # no second stage: "dw_partial" is the whole weight-gradient kernel
    us = {n: sum(v) / len(v) for n, v in samples.items()}
    us_median = {n: v[len(v) // 2] for n, v in samples.items()}
    us_min = {n: v[0] for n, v in samples.items()}
    step_samples = sorted(1e3 * e[0].elapsed_time(e[4]) for e in evs)

    # the same step with the fused backward call (reads dY once: 5 tensor passes instead of 6); reported beside
    # the headline number against its own algorithmic bytes, never as `value`
    fused = None
    if fused_on:
        for i in range(max(args.warmup, 8)):
            step_fused(sets[i % args.sets])
        torch.cuda.synchronize()
        f0 = torch.cuda.Event(enable_timing=True); f1 = torch.cuda.Event(enable_timing=True)
        f0.record()
        for i in range(args.steps):
            step_fused(sets[i % args.sets])
        f1.record()
        torch.cuda.synchronize()
        fused_ms = f0.elapsed_time(f1) / args.steps
        fevs = new_events(n_ev, 3)
        for i in range(n_ev):
            step_fused(sets[i % args.sets], fevs[i])
        torch.cuda.synchronize()
        fb = sorted(1e3 * e[1].elapsed_time(e[2]) for e in fevs)
        fused = {"us_per_step": round(fused_ms * 1e3, 2),
                 "fwd_us": round(1e3 * sum(e[0].elapsed_time(e[1]) for e in fevs) / n_ev, 2),
                 "bwd_us": round(sum(fb) / n_ev, 2), "bwd_us_median": round(fb[n_ev // 2], 2),
                 "bwd_us_min": round(fb[0], 2)}

    es = wl.elem_size
    step_bytes = algorithmic_bytes(wl.B, wl.C, wl.L, K, es, "step")
    path_bytes = algorithmic_bytes(wl.B, wl.C, wl.L, K, es, "fwd")
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    dom = max(("fwd", "dx", "dw_partial"), key=lambda n: us[n])
    achieved = path_bytes / (us[dom] * 1e-6) / 1e9
    flops = in_range_flops(wl.B, wl.C, wl.L, K, p)
    out = {
        "metric": "effective HBM GB/s per fwd+dX+dW step (and us per step), B32 C256 L4096 K64 fp32"
                  if args.workload == 1 else f"effective HBM GB/s per fwd+dX+dW step, {wl.name}",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "us_per_step": round(ms_per_step * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "C": wl.C, "L": wl.L, "K": K, "pad_left": p,
                   "storage": wl.dtype, "buffer_sets": args.sets, "dw_single_kernel": bool(single),
                   "step_algorithmic_bytes": step_bytes, "path_algorithmic_bytes": path_bytes,
                   "path_flops_in_range": flops, "path_flops_dense": dense_flops(wl.B, wl.C, wl.L, K)},
        "paths_us": {n: round(v, 2) for n, v in us.items()},
        "paths_us_median": {n: round(v, 2) for n, v in us_median.items()},
        "paths_us_min": {n: round(v, 2) for n, v in us_min.items()},
        "step_us_from_events": {"mean": round(sum(step_samples) / len(step_samples), 2),
                                "median": round(step_samples[len(step_samples) // 2], 2),
                                "min": round(step_samples[0], 2), "samples": len(step_samples)},
        "input_values": args.data,
        "sclk_mhz_during_timed_steps": ({"samples": len(clocks), "min": min(clocks), "median": sorted(clocks)[len(clocks) // 2],
                                         "max": max(clocks)} if clocks else None),
        "warmup_steps_run": warm_done, "warmup_seconds": round(warm_seconds, 3),
        "first_steps_us": first_steps_us,
        "paths_gbps": {"fwd": round(path_bytes / us["fwd"] / 1e3, 1), "dx": round(path_bytes / us["dx"] / 1e3, 1),
                       "dw": round(path_bytes / (us["dw_partial"] + us["dw_finalize"]) / 1e3, 1)},
        "paths_frac_of_hbm_peak": {"fwd": round(path_bytes / us["fwd"] / 1e3 / HBM_PEAK_GBPS, 4),
                                   "dx": round(path_bytes / us["dx"] / 1e3 / HBM_PEAK_GBPS, 4),
                                   "dw": round(path_bytes / (us["dw_partial"] + us["dw_finalize"]) / 1e3 / HBM_PEAK_GBPS, 4)},
        "paths_tflops": {n: round(flops / us[n] / 1e6, 2) for n in ("fwd", "dx", "dw_partial")},
        "roofline": None,
    }
    # The roof that binds the dominant kernel is the one it sits closest to: HBM (algorithmic bytes) or,
    # for filters as long as the sequence, the matrix peak of the storage type (in-range flops).
    hbm_frac = achieved / HBM_PEAK_GBPS
    tflops = flops / us[dom] / 1e6
    mfma_peak = MFMA_F32_PEAK_TFLOPS if wl.dtype == "f32" else MFMA_BF16_PEAK_TFLOPS
    mfma_frac = tflops / mfma_peak
    # HBM bytes per launch of the dominant kernel from the committed counter summary, if one exists and the kernel's
    # sources have not changed since (a stale figure is withheld)
    tm = measured_traffic(args.workload, dom)
    traffic = tm[0] if tm and not tm[2] else None
    traffic_note = ({"profile": tm[1], "stale": tm[2]} if tm else None)
    if hbm_frac >= mfma_frac:
        out["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                           "unit": "GB/s", "frac": round(hbm_frac, 4), "traffic": traffic,
                           "traffic_from": traffic_note, "kernel_us": round(us[dom], 2),
                           "kernel_us_median": round(us_median[dom], 2), "kernel_us_min": round(us_min[dom], 2),
                           "algorithmic_bytes": path_bytes}
    else:
        out["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": round(tflops, 2), "peak": mfma_peak,
                           "unit": "TFLOP/s", "frac": round(mfma_frac, 4), "traffic": traffic,
                           "traffic_from": traffic_note, "kernel_us": round(us[dom], 2),
                           "kernel_us_median": round(us_median[dom], 2), "kernel_us_min": round(us_min[dom], 2),
                           "algorithmic_flops": flops}
    if fused:
        n_elems = wl.B * wl.C * wl.L
        fused_step_bytes = (5 * n_elems + 3 * wl.C * K) * es        # fwd 2N + CK, fused backward 3N + 2CK
        fused_bwd_bytes = (3 * n_elems + 2 * wl.C * K) * es
        fused["step_algorithmic_bytes"] = fused_step_bytes
        fused["step_gbps"] = round(fused_step_bytes / (fused["us_per_step"] * 1e-6) / 1e9, 1)
        fused["bwd_gbps"] = round(fused_bwd_bytes / (fused["bwd_us"] * 1e-6) / 1e9, 1)
        fused["bwd_frac_of_hbm_peak"] = round(fused["bwd_gbps"] / HBM_PEAK_GBPS, 4)
        fused["speedup_vs_three_calls"] = round(ms_per_step * 1e3 / fused["us_per_step"], 3)
        tb = measured_traffic(args.workload, "bwd_fused")
        fused["bwd_traffic"] = tb[0] if tb and not tb[2] else None
        out["fused_backward"] = fused
    # the achievable ceiling beside the published peak: a plain device copy of 1 GiB, which nothing caches
    del sets
    torch.cuda.empty_cache()
    cr = measure_copies((1024,))["1024MiB"]
    out["copy_roof"] = {"GBps": cr["GBps"], "frac_of_hbm_peak": round(cr["GBps"] / HBM_PEAK_GBPS, 4),
                        "what": "plain device copy of 1 GiB (read + write), 20 back to back"}
    out["paths_frac_of_copy_roof"] = {k: round(v / cr["GBps"], 4) for k, v in out["paths_gbps"].items()}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, inputs)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
