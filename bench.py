#!/usr/bin/env python3
"""Benchmark of the fused spectral convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3] [--no-extras]

A step is one pass of the whole hot path (load, pruned forward FFT, truncation, CGEMM over the hidden
dimension, zero padding, pruned inverse FFT, store) over one batch of synthetic input that is already
resident in HBM.  The default workload is the 1-D production shape (B=256, C=128, N=1024, K=128).
Successive steps rotate through a pool of identical (x, y) buffer pairs larger than the last-level cache, so
every step reads its input from HBM and no step overwrites output lines still cached from an earlier one.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X published dense BF16 matrix rate
BF16_PRODUCTS = 6               # BF16 products per FP32 multiply-add of the exact three-term operand split


def roofline_of(w, dev):
    """Which roofline bounds the layer and the fraction reached, from the device seconds per layer `dev`.
    Memory floor: the algorithmic bytes at the HBM peak.  Matrix floor: the contraction flops on the pipe the kernels
    run them on, the BF16 matrix pipe with six BF16 products per FP32 product (so its FP32-equivalent peak is
    2.5 PFLOP/s / 6).  The larger floor is the bound; a layer whose bytes would take under 5 us at the HBM peak is
    bound by launch and pipeline latency and its fractions say nothing about the kernel."""
    t_hbm = w.compulsory_bytes / (HBM_PEAK_GBPS * 1e9)
    t_mfma = flops_of(w) * BF16_PRODUCTS / (BF16_MFMA_PEAK_TFLOPS * 1e12)
    bound = "latency" if t_hbm < 5e-6 else "mfma_bf16x3" if t_mfma > t_hbm else "hbm"
    return {"bound": bound, "frac": max(t_hbm, t_mfma) / dev,
            "hbm_frac": t_hbm / dev, "bf16_pipe_frac": t_mfma / dev,
            "flop_per_byte": flops_of(w) / w.compulsory_bytes,
            "effective_hbm_GBps": w.compulsory_bytes / dev / 1e9,
            "contraction_TFLOPs": flops_of(w) / dev / 1e12}


def pick_config(name: str):
    from paper_2504_11681_amd import inputs
    table = {"cfg1": inputs.CONFIGS[0], "cfg2": inputs.CONFIGS[1], "cfg3": inputs.CONFIGS[2], "cfg4": inputs.CONFIGS[3]}
    for w in inputs.sweep_configs():
        table[w.name] = w
    if name not in table:
        raise SystemExit(f"unknown config {name!r}; choose from {sorted(table)}")
    return table[name]


def device_inputs(w, torch):
    """Seeded inputs of the workload, generated on the host and moved to HBM before timing starts."""
    from paper_2504_11681_amd import inputs
    xd = torch.empty((w.B, w.C_in) + w.spatial, dtype=torch.complex64, device="cuda")
    for b in range(w.B):
        xd[b] = torch.from_numpy(inputs.make_x_element(w.seed, b, w.C_in, w.spatial)).cuda()
    Wd = torch.from_numpy(inputs.make_W(w.seed, w.C_in, w.C_out)).cuda()
    yd = torch.zeros((w.B, w.C_out) + w.spatial, dtype=torch.complex64, device="cuda")
    return xd, Wd, yd


RAMP_SECONDS = 0.3   # the engine clock needs ~0.1 s of continuous work to climb from its idle state to the sustained one


def time_calls(torch, fn, steps: int, warmup: int, ramp: float = RAMP_SECONDS):
    """Returns (wall seconds for `steps` calls, mean per-call device time in seconds from HIP events
    recorded on the stream the kernels are launched on).

    Before the `warmup` untimed calls the same call is repeated for `ramp` seconds: a GPU that has been idle sits
    in a low-power state (engine clock near 100 MHz) and reaches its sustained clock (about 2.25 GHz under this
    load) only after some tens of milliseconds of work, so a short run started from idle reports the clock ramp,
    not the kernel (measured: 139 us per layer over 60 calls from idle, 119 us sustained)."""
    t_end = time.perf_counter() + ramp
    while time.perf_counter() < t_end:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev = e0.elapsed_time(e1) / steps * 1e-3     # back-to-back launches on one stream
    return wall, dev


def per_call_stats(torch, fn, n: int = 100):
    """Median and minimum device time of single calls (seconds), each bracketed by its own pair of HIP events on the
    launch stream; run right after the timed region, so the clock is still at its sustained value."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) * 1e-3 for a, b in ev)
    return t[len(t) // 2], t[0]


def flops_of(w):
    """Contraction flops on the retained modes (8 real flops per complex MAC)."""
    return 8.0 * w.B * (w.K ** w.dims) * w.C_in * w.C_out


def transform_flops_of(w):
    """Estimate of the real flops of the pruned transforms: per pencil N/K sub-transforms of length K plus one pruned
    radix-N/K combine, 5 N log2 K + 8 K (N/K - 1), for the B (C_in + C_out) pencils of the last axis and, in 2-D, N
    pencils per image on the first-axis pass of the forward side and K on the other (mirrored on the inverse side)."""
    import math
    per_pencil = 5.0 * w.N * math.log2(w.K) + 8.0 * w.K * (w.N / w.K - 1)
    images = w.B * (w.C_in + w.C_out)
    return images * per_pencil * (1 if w.dims == 1 else (w.N + w.K))


def buffer_sets(w):
    """Number of (x, y) buffer pairs the timed launches rotate through: enough that one round of the pool is
    at least 1 GiB, four times the 256 MB last-level cache, so that no launch finds its input or the lines of
    its output left there by an earlier launch."""
    pair = 16 * w.B * (w.C_in + w.C_out) * (w.N ** w.dims) // 2
    return max(2, min(64, -(-(1 << 30) // pair)))


def graph_time(w, torch, binding, launches=50, replays=40):
    """Device time per layer when `launches` fused calls are captured once in a HIP graph and the graph is replayed:
    what a launch-bound shape costs inside a captured loop.  Every replay is checked against the eager result."""
    xd, Wd, yd = device_inputs(w, torch)
    fn = getattr(binding, "spectral_conv%dd" % w.dims)
    binding.ensure_workspace(binding.workspace_bytes(w.dims, 0, w.B, w.C_in, w.C_out, w.N, w.K), xd.device)
    fn(xd, Wd, yd, w.K)                                   # eager: first-call setup happens outside the capture
    torch.cuda.synchronize()
    want = yd.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn(xd, Wd, yd, w.K, side.cuda_stream)
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for _ in range(launches):
                fn(xd, Wd, yd, w.K, torch.cuda.current_stream().cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    ok = True
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(5):
        yd.zero_()
        g.replay()
        torch.cuda.synchronize()
        ok = ok and bool(torch.equal(yd, want))
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    dt = e0.elapsed_time(e1) * 1e-3 / (replays * launches)
    del g, xd, Wd, yd, want
    torch.cuda.empty_cache()
    return dt, ok


VARIANT_SUFFIX = ("", "_staged", "_pruned", "_fft_gemm", "_gemm_ifft", "_auto")


def measure(w, torch, binding, steps, warmup, staged=False, pruned=False, ramp=RAMP_SECONDS, variant=None,
            stats=None):
    """variant: 0 fused, 1 staged (five kernels), 2 pruned (three kernels), 3 FFT+CGEMM fused, 4 CGEMM+iFFT fused,
    5 per-shape dispatch."""
    xd, Wd, yd = device_inputs(w, torch)
    sets = [(xd, yd)] + [(xd.clone(), torch.zeros_like(yd)) for _ in range(buffer_sets(w) - 1)]
    if variant is None:
        variant = 2 if pruned else 1 if staged else 0
    name = ("spectral_conv%dd" % w.dims) + VARIANT_SUFFIX[variant]
    fn = getattr(binding, name)
    binding.ensure_workspace(binding.workspace_bytes(w.dims, variant, w.B, w.C_in, w.C_out, w.N, w.K), xd.device)
    stream = torch.cuda.current_stream().cuda_stream
    turn = [0]

    def call():
        xi, yi = sets[turn[0] % len(sets)]
        turn[0] += 1
        fn(xi, Wd, yi, w.K, stream)

    wall, dev = time_calls(torch, call, steps, warmup, ramp)
    if stats is not None:
        stats["median_s"], stats["min_s"] = per_call_stats(torch, call)
    del xd, Wd, yd, sets
    torch.cuda.empty_cache()
    return wall, dev


def measure_strips(w, torch, binding, steps, warmup, ramp):
    """Device seconds per layer of the paper's own 2-D pipeline (tfno_spectral_conv2d_strips: first-axis FFT with
    truncation, fused 1-D kernel on the retained rows, first-axis iFFT with padding) on the 2-D workload w."""
    xd, Wd, yd = device_inputs(w, torch)
    sets = [(xd, yd), (xd.clone(), torch.zeros_like(yd))]
    binding.ensure_workspace(binding.workspace_bytes_2d(7, w.B, w.C_in, w.C_out, w.N, w.N, w.K, w.K), xd.device)
    stream = torch.cuda.current_stream().cuda_stream
    turn = [0]

    def call():
        xi, yi = sets[turn[0] % 2]
        turn[0] += 1
        binding.spectral_conv2d_strips(xi, Wd, yi, w.K, w.K, stream)

    _, dev = time_calls(torch, call, steps, warmup, ramp)
    del xd, Wd, yd, sets
    torch.cuda.empty_cache()
    return dev


def measure_rect(torch, binding, B, C, N1, N2, K1, K2, steps, warmup, ramp):
    """Device seconds per layer of the non-square 2-D entry point on seeded inputs of the usual recipe."""
    from paper_2504_11681_amd import inputs
    seed = 6
    xd = torch.empty((B, C, N1, N2), dtype=torch.complex64, device="cuda")
    for b in range(B):
        xd[b] = torch.from_numpy(inputs.make_x_element(seed, b, C, (N1, N2))).cuda()
    Wd = torch.from_numpy(inputs.make_W(seed, C, C)).cuda()
    pair = 16 * B * C * N1 * N2
    nsets = max(2, min(64, -(-(1 << 30) // pair)))
    sets = [(xd, torch.zeros_like(xd))] + [(xd.clone(), torch.zeros_like(xd)) for _ in range(nsets - 1)]
    binding.ensure_workspace(binding.workspace_bytes_2d(0, B, C, C, N1, N2, K1, K2), xd.device)
    stream = torch.cuda.current_stream().cuda_stream
    turn = [0]

    def call():
        xi, yi = sets[turn[0] % len(sets)]
        turn[0] += 1
        binding.spectral_conv2d_rect(xi, Wd, yi, K1, K2, stream)

    _, dev = time_calls(torch, call, steps, warmup, ramp)
    del xd, Wd, sets
    torch.cuda.empty_cache()
    return dev


def measure_permode(torch, binding, w, steps, warmup, ramp):
    """Device seconds per layer of the per-mode-weight entry point on workload w (W drawn per mode with the usual
    recipe), and the bytes a layer must move (x, y and the weight tensor once)."""
    from paper_2504_11681_amd import inputs
    xd, _, yd = device_inputs(w, torch)
    modes = w.K ** w.dims
    Wd = torch.from_numpy(inputs.make_W(w.seed, w.C_in, w.C_out * modes)).cuda().reshape((w.C_in, w.C_out) + (w.K,) * w.dims)
    sets = [(xd, yd)] + [(xd.clone(), torch.zeros_like(yd)) for _ in range(buffer_sets(w) - 1)]
    fn = binding.spectral_conv1d_permode if w.dims == 1 else binding.spectral_conv2d_permode
    stream = torch.cuda.current_stream().cuda_stream
    turn = [0]

    def call():
        xi, yi = sets[turn[0] % len(sets)]
        turn[0] += 1
        fn(xi, Wd, yi, stream)

    _, dev = time_calls(torch, call, steps, warmup, ramp)
    nbytes = 8 * w.B * (w.N ** w.dims) * (w.C_in + w.C_out) + 8 * w.C_in * w.C_out * modes
    del xd, Wd, yd, sets
    torch.cuda.empty_cache()
    return dev, nbytes


def measure_real(torch, binding, w, steps, warmup, ramp):
    """Device seconds per layer of the real-valued entry point on the shape of workload w (x = real parts of the
    seeded inputs), and its compulsory bytes (float32 x and y once)."""
    xd, Wd, yd = device_inputs(w, torch)
    xr = xd.real.contiguous()
    yr = torch.zeros(yd.shape, dtype=torch.float32, device="cuda")
    del xd, yd
    pair = 4 * w.B * (w.C_in + w.C_out) * w.N
    nsets = max(2, min(64, -(-(1 << 30) // pair)))
    sets = [(xr, yr)] + [(xr.clone(), torch.zeros_like(yr)) for _ in range(nsets - 1)]
    stream = torch.cuda.current_stream().cuda_stream
    turn = [0]

    def call():
        xi, yi = sets[turn[0] % len(sets)]
        turn[0] += 1
        binding.spectral_conv1d_real(xi, Wd, yi, w.K, stream)

    _, dev = time_calls(torch, call, steps, warmup, ramp)
    del xr, yr, Wd, sets
    torch.cuda.empty_cache()
    return dev, pair + 8 * w.C_in * w.C_out


def measure_fno2d(torch, binding, B, C, N1, N2, M1, M2, steps, warmup, ramp):
    """Device seconds per layer of the real-field 2-D FNO layer and its compulsory bytes; inputs of the usual recipe
    (real parts), weights per mode."""
    from paper_2504_11681_amd import inputs
    seed = 9
    xd = torch.empty((B, C, N1, N2), dtype=torch.float32, device="cuda")
    for b in range(B):
        xd[b] = torch.from_numpy(inputs.make_x_element(seed, b, C, (N1, N2)).real.copy()).cuda()
    Wd = torch.from_numpy(inputs.make_W(seed, C, C * 2 * M1 * M2)).cuda().reshape(C, C, 2 * M1, M2).contiguous()
    pair = 8 * B * C * N1 * N2
    nsets = max(2, min(64, -(-(1 << 30) // pair)))
    sets = [(xd, torch.zeros_like(xd))] + [(xd.clone(), torch.zeros_like(xd)) for _ in range(nsets - 1)]
    stream = torch.cuda.current_stream().cuda_stream
    turn = [0]

    def call():
        xi, yi = sets[turn[0] % len(sets)]
        turn[0] += 1
        binding.fno2d_real(xi, Wd, yi, stream)

    _, dev = time_calls(torch, call, steps, warmup, ramp)
    del xd, Wd, sets
    torch.cuda.empty_cache()
    return dev, pair + 8 * C * C * 2 * M1 * M2


def cpu_baseline(w):
    """The float64 oracle, as it stands, timed on the host cores over the whole workload (1-D) or
    over a bounded sample of batch elements (2-D)."""
    import numpy as np
    import oracle
    from paper_2504_11681_amd import inputs
    oracle.build()
    nb = w.B if w.dims == 1 else min(w.B, 4)
    x = np.stack([inputs.make_x_element(w.seed, b, w.C_in, w.spatial) for b in range(nb)])
    W = inputs.make_W(w.seed, w.C_in, w.C_out)
    fn = oracle.spectral_conv1d if w.dims == 1 else oracle.spectral_conv2d
    reps = 0
    t0 = time.perf_counter()
    while reps < 3 or (time.perf_counter() - t0 < 1.0 and reps < 20):    # about 15-30 core-seconds in all
        _, used = fn(x, W, w.K)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": (nb / w.B) / dt, "unit": "layers/s", "cores": int(used), "kind": "oracle",
            "sample": f"{nb} of {w.B} batch elements of {w.name}, float64, mean of {reps} passes, {dt:.2f} s wall "
                      f"each on {int(used)} threads; layers/s scaled by {nb}/{w.B}"}


def stream_copy_rate(torch, nbytes, steps=200):
    """What the machine streams when it reads and writes at the same time, as the fused layer does: a plain
    device-to-device copy of `nbytes` (torch's copy_, i.e. the runtime's copy kernel) through rotating buffer pairs
    totalling at least 1 GiB, timed with events like the layers.  Context for roofline.frac, not part of the path."""
    sets = max(2, -(-(1 << 30) // (2 * nbytes)))
    src = [torch.ones(nbytes, dtype=torch.uint8, device="cuda") for _ in range(sets)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(sets)]
    for i in range(20):
        dst[i % sets].copy_(src[i % sets])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        dst[i % sets].copy_(src[i % sets])
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) / 1e3 / steps
    del src, dst
    torch.cuda.empty_cache()
    return {"kernel": "device-to-device copy (reads and writes at once)", "bytes_read": nbytes, "bytes_written": nbytes,
            "us_per_copy": sec * 1e6, "GBps": 2 * nbytes / sec / 1e9, "frac_of_peak": 2 * nbytes / sec / 1e9 / HBM_PEAK_GBPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--variant", default="fused", choices=["fused", "staged", "pruned", "fft_gemm", "gemm_ifft", "auto"],
                    help="entry point timed as the main measurement (1-D workloads; default: the fused kernel)")
    ap.add_argument("--ramp", type=float, default=RAMP_SECONDS,
                    help="seconds of untimed calls before the warm-up steps that bring the engine clock from idle to "
                         "its sustained value (0 for counter-collection runs, where every launch is slow)")
    ap.add_argument("--no-extras", action="store_true", help="skip the staged, 2-D and CPU-baseline legs")
    ap.add_argument("--only", default=None, choices=["per_mode_weights", "real_1d"],
                    help="time just this layer on --config and print a short JSON line (for profiler runs of the "
                         "kernels behind the widened entry points): per_mode_weights = tfno_spectral_conv{1,2}d_permode, "
                         "real_1d = tfno_spectral_conv1d_real")
    ap.add_argument("--shape", default=None, metavar="B,C,N,K",
                    help="time the 1-D entry point chosen by --variant on this shape (C_in = C_out = C) instead of a named "
                         "configuration and print a short JSON line (for the short-pencil and small-batch shapes of the "
                         "profiles)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of one workload, time every cell of the hidden-dimension sweep (B=512, N=256, C in "
                         "{32,64,128,256}, K in {32,64,128}) with the fused kernel (the paper's variant D), the two "
                         "partially fused variants (B: FFT+CGEMM, C: CGEMM+iFFT), the unfused pruned variant (A) and the "
                         "five-kernel staged baseline, and print one JSON line with all cells")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy three times (reads 256 MiB, writes "
                         "256 MiB per launch): the known-size kernel that calibrates rocprofv3's FETCH_SIZE / "
                         "WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU (the path shards over the batch axis with no "
                         "exchange; no multi-GPU code exists). Run with --gpus 1.")

    import torch
    from paper_2504_11681_amd import binding
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs the MI355X (no CPU fallback exists)")
    binding.lib()

    if args.copy_probe:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.sweep:
        from paper_2504_11681_amd import inputs
        cells = []
        for w in inputs.sweep_configs():
            _, dev = measure(w, torch, binding, args.steps, args.warmup, ramp=args.ramp)
            _, pdev = measure(w, torch, binding, args.steps, args.warmup, pruned=True, ramp=args.ramp)
            _, bdev = measure(w, torch, binding, args.steps, args.warmup, variant=3, ramp=args.ramp)
            _, cdev = measure(w, torch, binding, args.steps, args.warmup, variant=4, ramp=args.ramp)
            _, adev = measure(w, torch, binding, args.steps, args.warmup, variant=5, ramp=args.ramp)
            _, sdev = measure(w, torch, binding, max(5, args.steps // 10), 2, staged=True, ramp=args.ramp)
            times = {"fused": dev, "pruned": pdev, "fft_gemm": bdev, "gemm_ifft": cdev}
            cells.append({"workload": w.name, "C": w.C_in, "K": w.K, "fused_us": dev * 1e6, "pruned_us": pdev * 1e6,
                          "fft_gemm_us": bdev * 1e6, "gemm_ifft_us": cdev * 1e6, "auto_us": adev * 1e6,
                          "staged_us": sdev * 1e6, "best": min(times, key=times.get),
                          "fused_hbm_frac": w.compulsory_bytes / dev / 1e9 / HBM_PEAK_GBPS,
                          "fused_contraction_TFLOPs": flops_of(w) / dev / 1e12,
                          "auto_roofline": roofline_of(w, adev)})
        print(json.dumps({"metric": "fused_vs_unfused_crossover", "unit": "us per layer (HIP events)", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "dtype": "f32", "data": "synthetic",
                          "cells": cells}), flush=True)
        return

    if args.shape:
        from paper_2504_11681_amd import inputs
        B, C, N, K = (int(v) for v in args.shape.split(","))
        w = inputs.Workload(f"shape_1d_B{B}_C{C}_N{N}_K{K}", 1, B, C, C, N, K, 0)
        vid = ["fused", "staged", "pruned", "fft_gemm", "gemm_ifft", "auto"].index(args.variant)
        _, dev = measure(w, torch, binding, args.steps, args.warmup, ramp=args.ramp, variant=vid)
        print(json.dumps({"metric": "us_per_layer", "workload": w.name, "entry_point": "tfno_spectral_conv1d" + VARIANT_SUFFIX[vid],
                          "us_per_layer": dev * 1e6, "steps": args.steps, "warmup": args.warmup,
                          "roofline": roofline_of(w, dev), "dtype": "f32", "data": "synthetic", "n_gpus": 1}), flush=True)
        return
    w = pick_config(args.config)
    if args.only:
        fn = measure_permode if args.only == "per_mode_weights" else measure_real
        devo, nbo = fn(torch, binding, w, args.steps, args.warmup, args.ramp)
        print(json.dumps({"metric": args.only, "workload": w.name, "us_per_layer": devo * 1e6, "steps": args.steps,
                          "warmup": args.warmup, "bytes_per_layer": nbo, "hbm_frac": nbo / devo / 1e9 / HBM_PEAK_GBPS,
                          "dtype": "f32", "data": "synthetic", "n_gpus": 1}), flush=True)
        return
    vid = ["fused", "staged", "pruned", "fft_gemm", "gemm_ifft", "auto"].index(args.variant)
    st = {}
    wall, dev = measure(w, torch, binding, args.steps, args.warmup, ramp=args.ramp, variant=vid, stats=st)
    ms_per_step = wall / args.steps * 1e3
    layers_per_s = args.steps / wall
    alg_bytes = w.compulsory_bytes
    tpath = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "traffic.json")

    def committed_traffic(name):
        """HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated) from the committed counter summary that
        covers the workload: read from profiles/traffic.json, NOT measured in this run (counters need the profiler)."""
        if not os.path.exists(tpath):
            return None, None
        e = json.load(open(tpath)).get(name, {})
        src = e.get("source")
        if src and e.get("kernel"):
            src += ", kernel " + e["kernel"]
        return e.get("hbm_bytes_per_launch"), src

    def roofline_entry(wk, devk, kernel, stats=None):
        r = roofline_of(wk, devk)
        traffic, src = committed_traffic(wk.name)
        if r["bound"] == "mfma_bf16x3":
            e = {"bound": "mfma", "achieved": flops_of(wk) * BF16_PRODUCTS / devk / 1e12, "peak": BF16_MFMA_PEAK_TFLOPS,
                 "unit": "TFLOP/s", "pipe": "BF16 MFMA, six BF16 products per FP32 multiply-add (exact three-term split)"}
        else:
            e = {"bound": "hbm", "achieved": wk.compulsory_bytes / devk / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s"}
        e.update({"frac": e["achieved"] / e["peak"], "traffic": traffic,
                  "traffic_source": None if traffic is None else f"{src} (committed rocprofv3 counter summary, not measured in this run)",
                  "kernel": kernel, "algorithmic_bytes_per_launch": wk.compulsory_bytes,
                  "algorithmic_flops_per_launch": flops_of(wk), "flop_per_byte": r["flop_per_byte"],
                  "hbm_frac": r["hbm_frac"], "bf16_pipe_frac": r["bf16_pipe_frac"], "avg_launch_ms": devk * 1e3})
        if r["bound"] == "latency":
            e["note"] = "under 5 us of bytes at the HBM peak: bound by launch and pipeline latency"
        if stats:
            e["median_launch_ms"], e["min_launch_ms"] = stats["median_s"] * 1e3, stats["min_s"] * 1e3
        return e

    kernel_1d = ("k_fused1d_sym (N = 1024, K in {64, 128}); N = 256: k_fused1d with four waves (one or two operand "
                 "tiles) or eight waves, k_fused1d_pp for C_out > 128 and K <= 64; k_fused1d_ws / k_fused1d otherwise")
    out = {
        "metric": "fused_spectral_conv_layers_per_s",
        "value": layers_per_s,
        "unit": "layers/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "buffer_sets": buffer_sets(w),
        "clock_ramp_s": args.ramp,
        "config": {"workload": w.name, "dims": w.dims, "B": w.B, "C_in": w.C_in, "C_out": w.C_out,
                   "N": w.N, "K": w.K, "seed": w.seed,
                   "entry_point": "tfno_spectral_conv%dd" % w.dims + VARIANT_SUFFIX[vid]},
        # the same bytes over the wall-clock time per step (launch overhead included): the headline fraction
        "effective_hbm_GBps": alg_bytes / (wall / args.steps) / 1e9,
        "effective_hbm_frac_of_peak": alg_bytes / (wall / args.steps) / 1e9 / HBM_PEAK_GBPS,
        "contraction_TFLOPs": flops_of(w) / dev / 1e12,
        # secondary check: the butterflies against the FP32 vector rate this pool allows (packed FP32 is switched
        # off, so a CU array issues 78.6 TFLOP/s of FMAs, half the published 157.3)
        "transform_TFLOPs": transform_flops_of(w) / dev / 1e12,
        "transform_frac_of_unpacked_fp32_vector_peak": transform_flops_of(w) / dev / 1e12 / 78.6,
        "roofline": roofline_entry(w, dev, kernel_1d if w.dims == 1 else "tfno_spectral_conv2d (k_fwd2d, k_cgemm_modes, k_inv2d)", st),
    }

    if not args.no_extras:
        out["stream_copy"] = stream_copy_rate(torch, alg_bytes // 2)
        out["stream_copy"]["fused_time_over_copy_time"] = (
            (wall / args.steps) / (alg_bytes / (out["stream_copy"]["GBps"] * 1e9)))
        s_steps = max(5, args.steps // 10)
        swall, sdev = measure(w, torch, binding, s_steps, 2, staged=True, ramp=args.ramp)
        out["staged"] = {"ms_per_step": swall / s_steps * 1e3, "layers_per_s": s_steps / swall,
                         "variant": "five kernels: full FFT, truncate copy, CGEMM, pad copy, full iFFT (written for "
                                    "generality, not speed: not the fair unfused reference, see unfused_pruned)",
                         "fused_speedup": (swall / s_steps) / (wall / args.steps)}
        if w.dims == 1:
            # the paper's variant A: the same pruned transforms and the same matrix-pipe contraction as three kernels,
            # the truncated spectra crossing HBM -- the fair fused-versus-unfused ratio
            a_steps = max(20, args.steps // 4)
            awall, adev = measure(w, torch, binding, a_steps, max(5, args.warmup // 4), ramp=args.ramp, variant=2)
            out["unfused_pruned"] = {"ms_per_step": awall / a_steps * 1e3, "layers_per_s": a_steps / awall,
                                     "us_per_layer": adev * 1e6,
                                     "variant": "three kernels (tfno_spectral_conv1d_pruned): pruned FFT with built-in "
                                                "truncation, CGEMM, pruned iFFT with built-in padding",
                                     "fused_speedup": adev / dev}
        if w.name.startswith("cfg3"):
            w4 = pick_config("cfg4")
            steps4 = max(10, args.steps // 4)
            wall4, dev4 = measure(w4, torch, binding, steps4, 5, ramp=args.ramp)
            out["cfg4_2d"] = {"workload": w4.name, "steps": steps4, "ms_per_step": wall4 / steps4 * 1e3,
                              "layers_per_s": steps4 / wall4,
                              "effective_hbm_GBps": w4.compulsory_bytes / (wall4 / steps4) / 1e9,
                              "effective_hbm_frac_of_peak": w4.compulsory_bytes / (wall4 / steps4) / 1e9 / HBM_PEAK_GBPS,
                              "roofline": roofline_entry(w4, dev4, "tfno_spectral_conv2d (k_fwd2d, k_cgemm_modes, k_inv2d)")}
            # Everything below widens the report beyond the headline workloads; a failure there is recorded, not fatal
            # to the line (the headline figures above are already measured).
            try:
                # the 2-D ablation: the paper's own pipeline (strips of K retained rows through HBM around the fused
                # 1-D kernel) against the image kernels above
                sdev = measure_strips(w4, torch, binding, max(5, steps4 // 25), 2, args.ramp / 3)
                out["cfg4_2d"]["paper_2d_pipeline"] = {
                    "entry_point": "tfno_spectral_conv2d_strips", "us_per_layer": sdev * 1e6,
                    "structure": "first-axis FFT with truncation, fused FFT-CGEMM-iFFT along the last axis on the K "
                                 "retained rows, first-axis iFFT with padding; two [B, C, K, N] strips cross HBM",
                    "image_kernels_speedup": sdev / dev4}
            except Exception as exc:                                    # pragma: no cover
                out["cfg4_2d"]["paper_2d_pipeline"] = {"error": repr(exc)}
            try:
                # the remaining configurations: the two small 1-D shapes on the fused entry point and the twelve cells
                # of the hidden-dimension sweep on the per-shape dispatch (all variants of the sweep: --sweep)
                from paper_2504_11681_amd import inputs
                others = []
                for wo in [pick_config("cfg1"), pick_config("cfg2")] + list(inputs.sweep_configs()):
                    vo = 5 if wo.name.startswith("cfg5") else 0
                    _, devo = measure(wo, torch, binding, max(50, args.steps // 4), max(10, args.warmup // 4),
                                      ramp=args.ramp / 3, variant=vo)
                    cell = {"workload": wo.name, "entry_point": "tfno_spectral_conv1d" + VARIANT_SUFFIX[vo],
                            "us_per_layer": devo * 1e6, "layers_per_s": 1.0 / devo}
                    cell.update(roofline_of(wo, devo))
                    others.append(cell)
                    if cell["bound"] == "latency":
                        gdt, gok = graph_time(wo, torch, binding)
                        cell["us_per_layer_in_hip_graph"] = gdt * 1e6
                        cell["hip_graph_replays_match_eager"] = gok
                out["other_configs"] = others
                # non-square 2-D grids (same image kernels, each axis with its own length and mode count)
                rect = []
                for (Br, Cr, N1, N2, K1, K2) in [(32, 64, 128, 256, 32, 64), (32, 64, 256, 128, 64, 32), (64, 64, 64, 256, 16, 64)]:
                    devr = measure_rect(torch, binding, Br, Cr, N1, N2, K1, K2, max(50, args.steps // 4),
                                        max(10, args.warmup // 4), args.ramp / 3)
                    nbytes = 16 * Br * Cr * N1 * N2
                    rect.append({"workload": f"rect_2d_B{Br}_C{Cr}_N{N1}x{N2}_K{K1}x{K2}", "us_per_layer": devr * 1e6,
                                 "layers_per_s": 1.0 / devr, "bound": "hbm", "effective_hbm_GBps": nbytes / devr / 1e9,
                                 "hbm_frac": nbytes / devr / 1e9 / HBM_PEAK_GBPS})
                out["rect_2d"] = rect
                # long pencils through the per-shape dispatch
                longp = []
                for (Bl, Cl, Nl, Kl) in [(64, 128, 4096, 512), (128, 128, 2048, 256)]:
                    wl = inputs.Workload(f"long_1d_B{Bl}_C{Cl}_N{Nl}_K{Kl}", 1, Bl, Cl, Cl, Nl, Kl, 7)
                    _, devl = measure(wl, torch, binding, max(50, args.steps // 8), max(10, args.warmup // 8),
                                      ramp=args.ramp / 3, variant=5)
                    cell = {"workload": wl.name, "entry_point": "tfno_spectral_conv1d_auto", "us_per_layer": devl * 1e6,
                            "layers_per_s": 1.0 / devl}
                    cell.update(roofline_of(wl, devl))
                    longp.append(cell)
                out["long_1d"] = longp
                # an own weight matrix per retained mode (three kernels)
                pm = []
                for wp in (w, w4) if w.name.startswith("cfg3") else ():
                    devp, nb = measure_permode(torch, binding, wp, max(50, args.steps // 8), max(10, args.warmup // 8), args.ramp / 3)
                    pm.append({"workload": wp.name + "_permode", "us_per_layer": devp * 1e6, "layers_per_s": 1.0 / devp,
                               "bound": "hbm", "effective_hbm_GBps": nb / devp / 1e9, "hbm_frac": nb / devp / 1e9 / HBM_PEAK_GBPS,
                               "contraction_TFLOPs": flops_of(wp) / devp / 1e12})
                out["per_mode_weights"] = pm
                # the 2-D FNO layer on real fields
                fno = []
                for (Bf, Cf, N1, N2, M1, M2) in [(32, 64, 256, 256, 16, 32), (256, 64, 64, 64, 12, 12)]:
                    devf, nbf = measure_fno2d(torch, binding, Bf, Cf, N1, N2, M1, M2, max(50, args.steps // 8),
                                              max(10, args.warmup // 8), args.ramp / 3)
                    fno.append({"workload": f"fno2d_real_B{Bf}_C{Cf}_N{N1}x{N2}_M{M1}x{M2}", "us_per_layer": devf * 1e6,
                                "layers_per_s": 1.0 / devf, "bound": "hbm", "effective_hbm_GBps": nbf / devf / 1e9,
                                "hbm_frac": nbf / devf / 1e9 / HBM_PEAK_GBPS})
                out["fno2d_real"] = fno
                # the 1-D FNO layer on real fields (pruned transforms around the per-mode contraction), cfg3's shape
                if w.name.startswith("cfg3"):
                    xr = torch.randn((w.B, w.C_in, w.N), device="cuda", dtype=torch.float32)
                    Wm = torch.view_as_complex(torch.randn((w.C_in, w.C_out, w.K, 2), device="cuda", dtype=torch.float32)) / (w.C_in ** 0.5)
                    yr = torch.zeros((w.B, w.C_out, w.N), device="cuda", dtype=torch.float32)
                    strm = torch.cuda.current_stream().cuda_stream
                    _, dev1 = time_calls(torch, lambda: binding.fno1d_real(xr, Wm, yr, strm), max(50, args.steps // 8),
                                         max(10, args.warmup // 8), args.ramp / 3)
                    nb1 = 4 * w.B * w.N * (w.C_in + w.C_out) + 8 * w.C_in * w.C_out * w.K
                    out["fno1d_real"] = [{"workload": f"fno1d_real_B{w.B}_C{w.C_in}_N{w.N}_M{w.K}", "us_per_layer": dev1 * 1e6,
                                          "layers_per_s": 1.0 / dev1, "bound": "hbm", "effective_hbm_GBps": nb1 / dev1 / 1e9,
                                          "hbm_frac": nb1 / dev1 / 1e9 / HBM_PEAK_GBPS}]
                    del xr, Wm, yr
                    torch.cuda.empty_cache()
                # real-valued layer (R2C / C2R semantics): half the bytes of the complex layer
                if w.name.startswith("cfg3"):
                    devr, nbr = measure_real(torch, binding, w, max(50, args.steps // 4), max(10, args.warmup // 4), args.ramp / 3)
                    out["real_1d"] = [{"workload": w.name + "_real", "us_per_layer": devr * 1e6, "layers_per_s": 1.0 / devr,
                                       "bound": "hbm", "effective_hbm_GBps": nbr / devr / 1e9, "hbm_frac": nbr / devr / 1e9 / HBM_PEAK_GBPS}]
            except Exception as exc:    # noqa: BLE001 - reported in the JSON line
                out["widened_report_error"] = repr(exc)
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    main()
