#!/usr/bin/env python3
"""Benchmark of the frequency-domain convolution hot path on one MI355X.

One step = fprop + bprop + accGrad of the headline layer (S=128, f=f'=64, 27x27 input,
5x5 kernel, 32x32 Fourier basis) as the two calls fft_conv_fprop_save + fft_conv_backward:
six kernel launches (x, w and gy are transformed once each, the two backward contractions
share a launch and so do the inverse transforms of the two gradients).  Inputs are seeded synthetic fp32 tensors
already resident in device memory.  `extra` holds the same step as three independent passes,
on the library's own Fourier basis, the other configurations, tiled layers, the FFT sweep.

Prints ONE JSON line: effective TFLOP/s (direct-convolution FLOP count over measured time),
the roofline of the dominant kernel (durations from HIP events recorded by the library on its
own stream around each stage), and the fp64 CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix, published

STAGES = ("fft", "contraction", "ifft")   # kernels of one pass, in launch order

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch,
# scaled by what the same counters read for a plain 256 MiB copy: x2.00 and x1.00); the runs
# and the table are in profiles/c2_hbm_traffic.md.  Keyed by workload, then "pass.stage".
MEASURED_TRAFFIC_BYTES = {
    "C2": {   # keys: the launches of the fprop_save + backward step (paired or separate contractions)
        "fprop.fft": (1.205e4 * 2.0 + 5.225e4) * 1024,
        "fprop.contraction": (2.625e4 * 2.0 + 3.483e4) * 1024,
        "fprop.ifft": (1.748e4 * 2.0 + 1.693e4) * 1024,
        "backward.fft": (8.610e3 * 2.0 + 3.487e4) * 1024,
        "bprop.contraction": (2.617e4 * 2.0 + 3.482e4) * 1024,
        "backward.contraction": (5.572e4 * 2.0 + 5.313e4) * 1024,
        "bprop.ifft": (1.748e4 * 2.0 + 2.333e4) * 1024,
        "accgrad.contraction": (3.489e4 * 2.0 + 1.741e4) * 1024,
        "accgrad.ifft": (8.778e3 * 2.0 + 4.00e2) * 1024,
        "backward.ifft": (2.619e4 * 2.0 + 2.373e4) * 1024,
    },
}


def stage_model(cfg, pass_name):
    """Algorithmic bytes (FFT stages) and executed flops (contraction) of one pass."""
    S, f, fo, h, w, kh, kw, N = (cfg[k] for k in ("S", "f", "fo", "h", "w", "kh", "kw", "N"))
    oh, ow = h - kh + 1, w - kw + 1
    bins = N * (N // 2 + 1)
    x = (S * f, h, w); wt = (fo * f, kh, kw); gy = (S * fo, oh, ow)
    if pass_name == "fprop":
        A, B, C, (M, Nn, K) = x, wt, gy, (S, fo, f)
    elif pass_name == "bprop":
        A, B, C, (M, Nn, K) = gy, wt, x, (S, f, fo)
    else:
        A, B, C, (M, Nn, K) = gy, x, wt, (fo, f, S)
    fwd = lambda t: t[0] * (4 * t[1] * t[2] + 8 * bins)
    return {
        "fft": {"bytes": fwd(A) + fwd(B)},
        "fft_a": {"bytes": fwd(A)},
        "fft_b": {"bytes": fwd(B)},
        # executed real flops: three real multiply-adds per complex one (Gauss's 3-multiplication
        # product), i.e. 6 M N K per bin; a plain 4-multiplication product would execute 8 M N K
        "contraction": {"flops": 6 * M * Nn * K * bins,
                        "bytes": 8 * bins * (A[0] + B[0] + C[0])},
        "ifft": {"bytes": C[0] * (8 * bins + 4 * C[1] * C[2])},
    }


def direct_flops(cfg):
    S, f, fo, h, w, kh, kw = (cfg[k] for k in ("S", "f", "fo", "h", "w", "kh", "kw"))
    return 2 * S * f * fo * kh * kw * (h - kh + 1) * (w - kw + 1)


def run_step(hd, t, cfg, passes, reuse=False, basis=None):
    """One step.  reuse=True: fft_conv_fprop_save + fft_conv_backward (x and w are transformed
    once, gy once); reuse=False: the three independent passes.  basis=None leaves the Fourier
    basis to the library (the smallest one that holds the image); a number names it (the *_tiled
    entry points: a basis that holds the whole image runs the untiled pipeline at that basis)."""
    dims = (cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    if reuse and len(passes) == 3:
        if basis is None:
            hd.fft_conv_fprop_save(t["x"], t["w"], t["saved"], y=t["y"])
            hd.fft_conv_backward(t["gy"], t["saved"], *dims, gx=t["gx"], gw=t["gw"])
        else:
            hd.fft_conv_fprop_save_tiled(t["x"], t["w"], basis, t["saved"], y=t["y"])
            hd.fft_conv_backward_tiled(t["gy"], t["saved"], *dims, basis, gx=t["gx"], gw=t["gw"])
        return
    if "fprop" in passes:
        if basis is None:
            hd.fft_conv_fprop(t["x"], t["w"], y=t["y"])
        else:
            hd.fft_conv_fprop_tiled(t["x"], t["w"], basis, y=t["y"])
    if "bprop" in passes:
        if basis is None:
            hd.fft_conv_bprop(t["gy"], t["w"], cfg["h"], cfg["w"], gx=t["gx"])
        else:
            hd.fft_conv_bprop_tiled(t["gy"], t["w"], cfg["h"], cfg["w"], basis, gx=t["gx"])
    if "accgrad" in passes:
        if basis is None:
            hd.fft_conv_accgrad(t["x"], t["gy"], gw=t["gw"])
        else:
            hd.fft_conv_accgrad_tiled(t["x"], t["gy"], basis, gw=t["gw"])


BASES = (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128)


def library_basis(cfg):
    """The basis the ordinary entry points use for an untiled layer: the smallest that holds the image."""
    return next(b for b in BASES if b >= max(cfg["h"], cfg["w"]))


def device_tensors(cfg, seed):
    import torch
    from paper_1412_7580_amd import synth
    x, w, gy = synth.conv_inputs(seed=seed, **cfg)
    t = {"x": torch.from_numpy(x).cuda(), "w": torch.from_numpy(w).cuda(), "gy": torch.from_numpy(gy).cuda()}
    t["y"] = torch.empty_like(t["gy"]); t["gx"] = torch.empty_like(t["x"]); t["gw"] = torch.empty_like(t["w"])
    return t, (x, w, gy)


def add_saved(hd, t, cfg, basis=None):
    import torch
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    n = hd.saved_bytes(*dims) if basis is None else hd.saved_bytes_tiled(*dims, basis)
    t["saved"] = torch.empty(n // 4, device="cuda", dtype=torch.float32)


def time_steps(hd, t, cfg, passes, steps, warmup, reuse=False, basis=None):
    import torch
    for _ in range(warmup):
        run_step(hd, t, cfg, passes, reuse, basis)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step(hd, t, cfg, passes, reuse, basis)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def profile_stages(hd, t, cfg, passes, steps, basis=None):
    """Average execution time (ms) of each kernel of each pass over `steps` repetitions, from the
    start/stop events the library attaches to every dispatch on its stream.
    Returns {pass: [fft, contraction, ifft]}."""
    import torch
    hd.set_profiling(True)
    acc = {p: [0.0] * 3 for p in passes}
    for _ in range(steps):
        for p in passes:
            run_step(hd, t, cfg, (p,), False, basis)
            ms = hd.last_kernel_ms()
            for i in range(3):
                acc[p][i] += ms[i]
    hd.set_profiling(False)
    torch.cuda.synchronize()
    return {p: [v / steps for v in acc[p]] for p in passes}


FPROP_KERNELS = ("fprop.fft", "fprop.contraction", "fprop.ifft")
# fft_conv_backward: five launches, or four when both contractions go out as one launch
# (and three when the two inverse transforms share a launch as well)
BACKWARD_KERNELS = {5: ("backward.fft", "bprop.contraction", "bprop.ifft", "accgrad.contraction", "accgrad.ifft"),
                    4: ("backward.fft", "backward.contraction", "bprop.ifft", "accgrad.ifft"),
                    3: ("backward.fft", "backward.contraction", "backward.ifft")}


def profile_reuse_step(hd, t, cfg, steps, basis=None):
    """Same for the two-call step with transform reuse: {kernel name: ms}."""
    import torch
    hd.set_profiling(True)
    acc = {}
    dims = (cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    for _ in range(steps):
        if basis is None:
            hd.fft_conv_fprop_save(t["x"], t["w"], t["saved"], y=t["y"])
        else:
            hd.fft_conv_fprop_save_tiled(t["x"], t["w"], basis, t["saved"], y=t["y"])
        a = hd.last_kernel_ms()
        if basis is None:
            hd.fft_conv_backward(t["gy"], t["saved"], *dims, gx=t["gx"], gw=t["gw"])
        else:
            hd.fft_conv_backward_tiled(t["gy"], t["saved"], *dims, basis, gx=t["gx"], gw=t["gw"])
        b = hd.last_kernel_ms()
        for k, v in zip(FPROP_KERNELS + BACKWARD_KERNELS[len(b)], a + b):
            acc[k] = acc.get(k, 0.0) + v
    hd.set_profiling(False)
    torch.cuda.synchronize()
    return {k: v / steps for k, v in acc.items()}


def cpu_baseline(cfg, host_inputs, budget_s=12.0):
    """fp64 oracle (as it stands, OpenMP over output planes) on the same inputs: whole passes
    when they are cheap, repeated until about budget_s of CPU work; otherwise a seeded sample
    of output planes of each pass, scaled by the plane fraction."""
    import numpy as np
    import oracle
    x, w, gy = host_inputs
    S, f, fo = cfg["S"], cfg["f"], cfg["fo"]
    per_pass = direct_flops(cfg)
    rng = np.random.default_rng(0)

    def run(name, sel):
        if name == "fprop":
            oracle.conv_fprop(x, w, sel)
        elif name == "bprop":
            oracle.conv_bprop(gy, w, cfg["h"], cfg["w"], sel)
        else:
            oracle.conv_accgrad(x, gy, sel)

    plan = {}
    for name, nplanes in (("fprop", S * fo), ("bprop", S * f), ("accgrad", fo * f)):
        k = min(nplanes, 64)
        sel = np.sort(rng.choice(nplanes, size=k, replace=False))
        t0 = time.perf_counter(); run(name, sel); dt = max(time.perf_counter() - t0, 1e-4)
        want = int(k * (budget_s / 3) / dt)
        plan[name] = (nplanes, min(nplanes, max(k, want)), max(1, min(50, want // nplanes)))
    done_flops, spent, parts = 0.0, 0.0, []
    for name, (nplanes, k, reps) in plan.items():
        sel = None if k == nplanes else np.sort(rng.choice(nplanes, size=k, replace=False))
        t0 = time.perf_counter()
        run(name, sel)
        one = max(time.perf_counter() - t0, 1e-4)
        reps = max(1, min(200, int(budget_s / 3 / one))) if k == nplanes else 1
        for _ in range(reps - 1):
            run(name, sel)
        dt = time.perf_counter() - t0
        done_flops += per_pass * reps * k / nplanes
        spent += dt
        parts.append(f"{name}: {k}/{nplanes} planes x{reps} in {dt:.2f}s")
    return {"value": round(done_flops / spent / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": "fp64 direct convolution oracle; " + "; ".join(parts)}


def fft_sweep(hd, max_bytes=1 << 28, reps=3, sizes=None, sizes_1d_only=(256,)):
    """Stand-alone FFT sweep: R2C then C2R of signals of n - 3 samples, input sized to 256 MiB,
    algorithmic GB/s.  Default sizes: those of the benchmark definition (8 ... 128) plus n = 256
    in 1-D, one size beyond it."""
    import torch
    from paper_1412_7580_amd import synth
    sizes = synth.FFT_SWEEP_SIZES if sizes is None else sizes
    out = {}
    for dim in (1, 2):
        for n in tuple(sizes) + (tuple(sizes_1d_only) if dim == 1 else ()):
            ni = n - 3
            B = max_bytes // (4 * ni ** dim)
            shape = (B, ni) if dim == 1 else (B, ni, ni)
            x = torch.randn(shape, device="cuda", dtype=torch.float32)
            nbins = (n // 2 + 1) * (1 if dim == 1 else n)
            X = torch.empty((B, n // 2 + 1, 2) if dim == 1 else (B, n, n // 2 + 1, 2), device="cuda")
            y = torch.empty_like(x)
            fwd = (lambda: hd.fft_r2c_1d(x, n, out=X)) if dim == 1 else (lambda: hd.fft_r2c_2d(x, n, out=X))
            inv = (lambda: hd.fft_c2r_1d(X, n, ni, out=y)) if dim == 1 else (lambda: hd.fft_c2r_2d(X, n, ni, ni, out=y))
            res = {}
            for name, fn in (("r2c", fwd), ("c2r", inv)):
                fn(); torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    fn()
                e1.record(); torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / reps
                byts = B * (4 * ni ** dim + 8 * nbins)
                res[name] = {"ms": round(ms, 4), "GBps": round(byts / ms / 1e6, 1)}
            out[f"{dim}d_n{n}"] = res
            del x, X, y
    return out


def graph_replay_c1(hd, reps=200):
    """The smallest configuration is launch-bound (three kernels of a few microseconds): time
    its fprop eagerly, as a captured HIP graph (caller-supplied workspace, so the call
    allocates nothing) and as the one-launch fused kernel."""
    import torch
    import paper_1412_7580_amd as pkg
    from paper_1412_7580_amd import synth
    cfg = {k: v for k, v in synth.CONV_CONFIGS["C1"].items() if k != "passes"}
    t, _ = device_tensors(cfg, synth.CONV_SEEDS["C1"])
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    ws = torch.empty(hd.workspace_bytes(pkg.FPROP, *dims) // 4, device="cuda", dtype=torch.float32)

    def call():
        hd.fft_conv_fprop(t["x"], t["w"], y=t["y"], ws=ws)

    def timed(fn):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps
    eager = timed(call)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    replay = timed(graph.replay)
    # the same fprop as ONE launch (fft_conv_fprop_fused, on weights transformed ahead)
    wf = hd.fft_conv_transform_weights(t["w"], cfg["h"], cfg["w"])
    fused = timed(lambda: hd.fft_conv_fprop_fused(t["x"], wf, cfg["fo"], cfg["kh"], cfg["kw"], y=t["y"]))
    # and the layer's bprop: ordinary call against the one-launch kernel
    gy = torch.empty_like(t["y"]).uniform_(-1, 1)
    gx = torch.empty_like(t["x"])
    dims = (cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    bprop = timed(lambda: hd.fft_conv_bprop(gy, t["w"], cfg["h"], cfg["w"], gx=gx))
    bfused = timed(lambda: hd.fft_conv_bprop_fused(gy, wf, *dims, gx=gx))
    return {"eager_us_per_fprop": round(eager * 1e6, 2), "graph_replay_us_per_fprop": round(replay * 1e6, 2),
            "fused_one_launch_us_per_fprop": round(fused * 1e6, 2),
            "eager_us_per_bprop": round(bprop * 1e6, 2), "fused_one_launch_us_per_bprop": round(bfused * 1e6, 2)}


def tiled_layers(hd, reps=10):
    """Tiling (Section 6 of the paper) on two layers: an image beyond the largest basis, which
    the ordinary entry points tile by themselves, a mid-size layer run untiled and tiled, and a
    layer between the two whose basis is also chosen by measurement (fftconv_autotune_basis).
    Timing only (uniform[-1,1) inputs drawn on the device from a fixed seed); parity of the
    tiled path is covered by the tests."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(6)

    def mk(*shape):
        return torch.rand(shape, device="cuda", generator=gen) * 2 - 1

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    out = {}
    S, f, fo, h, w, k = 16, 64, 64, 224, 224, 5
    x, wt, gy = mk(S, f, h, w), mk(fo, f, k, k), mk(S, fo, h - k + 1, w - k + 1)
    y, gx, gw = torch.empty_like(gy), torch.empty_like(x), torch.empty_like(wt)
    saved = torch.empty(hd.saved_bytes(S, f, fo, h, w, k, k) // 4, device="cuda", dtype=torch.float32)
    fl = 3 * 2.0 * S * f * fo * k * k * (h - k + 1) * (w - k + 1)

    def step():
        hd.fft_conv_fprop_save(x, wt, saved, y=y)
        hd.fft_conv_backward(gy, saved, f, h, w, k, k, gx=gx, gw=gw)
    sec = timed(step)
    out["S16_f64_f'64_224x224_k5"] = {"tile_basis": hd.tile_basis(h, w, k, k, 0), "ms_per_step": round(sec * 1e3, 4),
                                      "effective_TFLOPs": round(fl / sec / 1e12, 2),
                                      "calls": "fft_conv_fprop_save + fft_conv_backward (tile by themselves)"}
    del x, wt, gy, y, gx, gw, saved
    S, f, fo, h, w, k = 32, 96, 96, 55, 55, 5
    x, wt, gy = mk(S, f, h, w), mk(fo, f, k, k), mk(S, fo, h - k + 1, w - k + 1)
    y, gx, gw = torch.empty_like(gy), torch.empty_like(x), torch.empty_like(wt)
    fl = 3 * 2.0 * S * f * fo * k * k * (h - k + 1) * (w - k + 1)

    def untiled():
        hd.fft_conv_fprop(x, wt, y=y); hd.fft_conv_bprop(gy, wt, h, w, gx=gx); hd.fft_conv_accgrad(x, gy, gw=gw)

    def tiled():
        hd.fft_conv_fprop_tiled(x, wt, 0, y=y); hd.fft_conv_bprop_tiled(gy, wt, h, w, 0, gx=gx)
        hd.fft_conv_accgrad_tiled(x, gy, 0, gw=gw)
    su, st = timed(untiled), timed(tiled)
    out["S32_f96_f'96_55x55_k5"] = {"untiled_basis": 56, "untiled_ms_per_step": round(su * 1e3, 4),
                                    "untiled_effective_TFLOPs": round(fl / su / 1e12, 2),
                                    "tile_basis": hd.tile_basis(h, w, k, k, 0), "tiled_ms_per_step": round(st * 1e3, 4),
                                    "tiled_effective_TFLOPs": round(fl / st / 1e12, 2),
                                    "calls": "three independent passes each way"}
    del x, wt, gy, y, gx, gw
    # a layer whose untiled basis would be 112: the ordinary entry points tile it by themselves;
    # naming basis 128 runs the untiled pipeline (one 128x128 transform per image)
    S, f, fo, h, w, k = 16, 128, 128, 112, 112, 3
    x, wt, gy = mk(S, f, h, w), mk(fo, f, k, k), mk(S, fo, h - k + 1, w - k + 1)
    y, gx, gw = torch.empty_like(gy), torch.empty_like(x), torch.empty_like(wt)
    fl = 3 * 2.0 * S * f * fo * k * k * (h - k + 1) * (w - k + 1)

    def ordinary():
        hd.fft_conv_fprop(x, wt, y=y); hd.fft_conv_bprop(gy, wt, h, w, gx=gx); hd.fft_conv_accgrad(x, gy, gw=gw)

    def one_tile():
        hd.fft_conv_fprop_tiled(x, wt, 128, y=y); hd.fft_conv_bprop_tiled(gy, wt, h, w, 128, gx=gx)
        hd.fft_conv_accgrad_tiled(x, gy, 128, gw=gw)
    so, s1 = timed(ordinary), timed(one_tile)
    out["S16_f128_f'128_112x112_k3"] = {"tile_basis": hd.tile_basis(h, w, k, k, 0), "ms_per_step": round(so * 1e3, 4),
                                        "effective_TFLOPs": round(fl / so / 1e12, 2),
                                        "basis128_ms_per_step": round(s1 * 1e3, 4),
                                        "basis128_effective_TFLOPs": round(fl / s1 / 1e12, 2),
                                        "calls": "three independent passes; ordinary entry points (tile by themselves) "
                                                 "vs the untiled pipeline on basis 128"}
    # basis selection by measurement against the library's static estimate
    n_auto, ms_auto = hd.autotune_basis(x, wt, gy, y=y, gx=gx, gw=gw, reps=3)
    out["S16_f128_f'128_112x112_k3"]["autotuned_basis"] = n_auto
    out["S16_f128_f'128_112x112_k3"]["autotuned_ms_per_step"] = round(ms_auto, 4)
    return out


def table4_layers(hd, reps=10):
    """The five layer shapes of the paper's Table 4 (S = 128) on synthetic inputs, three
    independent passes each with the library's own choice of basis / tiling, next to the times
    the paper prints for its cuFFT-based implementation on a Tesla K40m (context: another
    machine, another decade; not a target)."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(7)
    layers = {   # name: (f, f', h = w, k, paper's cuFFT-convolution ms for fprop, bprop, accGrad)
        "L1": (3, 96, 128, 11, (80.98, 66.49, 69.63)),
        "L2": (64, 64, 64, 9, (46.44, 46.25, 47.03)),
        "L3": (128, 128, 32, 9, (17.77, 16.97, 17.00)),
        "L4": (128, 128, 16, 7, (4.88, 4.71, 4.70)),
        "L5": (384, 384, 13, 3, (21.35, 20.22, 21.26)),
    }
    out = {}
    S = 128
    for name, (f, fo, h, k, paper_ms) in layers.items():
        mk = lambda *shape: torch.rand(shape, device="cuda", generator=gen) * 2 - 1
        x, wt, gy = mk(S, f, h, h), mk(fo, f, k, k), mk(S, fo, h - k + 1, h - k + 1)
        y, gx, gw = torch.empty_like(gy), torch.empty_like(x), torch.empty_like(wt)
        calls = (lambda: hd.fft_conv_fprop(x, wt, y=y), lambda: hd.fft_conv_bprop(gy, wt, h, h, gx=gx),
                 lambda: hd.fft_conv_accgrad(x, gy, gw=gw))
        ms = []
        for fn in calls:
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            ms.append((time.perf_counter() - t0) / reps * 1e3)
        fl = 2.0 * S * f * fo * k * k * (h - k + 1) ** 2
        out[name] = {"shape": f"S=128 f={f} f'={fo} {h}x{h} k{k}",
                     "ms[fprop,bprop,accgrad]": [round(v, 4) for v in ms],
                     "effective_TFLOPs[fprop,bprop,accgrad]": [round(fl / (v * 1e-3) / 1e12, 1) for v in ms],
                     "paper_K40m_cuFFT_conv_ms[fprop,bprop,accgrad]": list(paper_ms)}
        del x, wt, gy, y, gx, gw
    return out


def weights_ahead(hd, reps=30):
    """fprop with the weight transform computed ahead (fft_conv_transform_weights once, then
    fft_conv_fprop_weights) against the ordinary fprop, on the shapes of C2..C4 (timing only)."""
    import torch
    from paper_1412_7580_amd import synth
    gen = torch.Generator(device="cuda").manual_seed(8)
    out = {}
    for name in ("C2", "C3", "C4"):
        c = synth.CONV_CONFIGS[name]
        mk = lambda *shape: torch.rand(shape, device="cuda", generator=gen) * 2 - 1
        x, wt = mk(c["S"], c["f"], c["h"], c["w"]), mk(c["fo"], c["f"], c["kh"], c["kw"])
        y = hd.fft_conv_fprop(x, wt)
        wf = hd.fft_conv_transform_weights(wt, c["h"], c["w"])
        us = []
        for fn in (lambda: hd.fft_conv_fprop(x, wt, y=y),
                   lambda: hd.fft_conv_fprop_weights(x, wf, c["fo"], c["kh"], c["kw"], y=y)):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            us.append(round((time.perf_counter() - t0) / reps * 1e6, 1))
        out[name] = {"fprop_us": us[0], "fprop_weights_ahead_us": us[1], "weights_MB": round(wf.numel() * 4 / 1e6, 1)}
        del x, wt, y, wf
    return out


def device_copy_bandwidth(reps=20):
    """Plain device-to-device copy of 256 MiB and 1 GiB (read + write bytes over time): what the
    memory system delivers to the simplest kernel, for reading the FFT stages' GB/s against."""
    import torch
    out = {}
    for mib in (256, 1024):
        a = torch.ones(mib * (1 << 20) // 4, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            b.copy_(a)
        e1.record(); torch.cuda.synchronize()
        out[f"{mib}MiB"] = round(2 * a.numel() * 4 / (e0.elapsed_time(e1) / reps) / 1e6, 1)
        del a, b
    return out


def conv_sweep_3x3(hd, reps=10):
    """The workload of the paper's comparison of fbfft against cuFFT inside the convolution
    (Section 5.4): 3x3 kernels, h = w in {13, 16, 27, 32, 57, 64}, S = f = f' in {16, 32, 64, 128},
    all three passes (here: fft_conv_fprop_save + fft_conv_backward, library's basis).  The paper
    reports only speed ratios over its cuFFT path for these; the table is ms per step and
    effective TFLOP/s on this chip."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(9)
    out = {}
    for hw in (13, 16, 27, 32, 57, 64):
        row = {}
        for n in (16, 32, 64, 128):
            mk = lambda *shape: torch.rand(shape, device="cuda", generator=gen) * 2 - 1
            x, wt, gy = mk(n, n, hw, hw), mk(n, n, 3, 3), mk(n, n, hw - 2, hw - 2)
            y, gx, gw = torch.empty_like(gy), torch.empty_like(x), torch.empty_like(wt)
            saved = torch.empty(hd.saved_bytes(n, n, n, hw, hw, 3, 3) // 4, device="cuda", dtype=torch.float32)

            def step():
                hd.fft_conv_fprop_save(x, wt, saved, y=y)
                hd.fft_conv_backward(gy, saved, n, hw, hw, 3, 3, gx=gx, gw=gw)
            for _ in range(3):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                step()
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / reps
            fl = 3 * 2.0 * n * n * n * 9 * (hw - 2) ** 2
            row[f"S=f=f'={n}"] = {"ms": round(sec * 1e3, 4), "effective_TFLOPs": round(fl / sec / 1e12, 2)}
            del x, wt, gy, y, gx, gw, saved
        out[f"{hw}x{hw}"] = row
    return out


def rectangular_layers(hd, reps=10):
    """Layers with non-square images (sides up to 32): the three passes on the rectangular basis
    the ordinary entry points choose, beside the same layer on the square basis of the larger
    side (named through the *_tiled calls).  us per three passes, kernels only."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(11)
    mk = lambda *shape: torch.rand(shape, device="cuda", generator=gen) * 2 - 1
    out = {}
    for (S, f, fo, h, w, kh, kw) in ((128, 96, 256, 27, 13, 5, 3), (128, 96, 256, 13, 27, 3, 5),
                                     (128, 64, 64, 16, 32, 3, 3), (128, 64, 64, 8, 32, 3, 3),
                                     (128, 64, 64, 32, 8, 3, 3), (128, 64, 64, 20, 24, 3, 3)):
        x, wt, gy = mk(S, f, h, w), mk(fo, f, kh, kw), mk(S, fo, h - kh + 1, w - kw + 1)
        y, gx, gw = torch.empty_like(gy), torch.empty_like(x), torch.empty_like(wt)
        nr, nc, _ = hd.layer_basis(h, w, kh, kw)
        n = max(nr, nc)

        def timed(step):
            for _ in range(3):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                step()
            torch.cuda.synchronize()
            return round((time.perf_counter() - t0) / reps * 1e6, 1)

        def rect():
            hd.fft_conv_fprop(x, wt, y=y); hd.fft_conv_bprop(gy, wt, h, w, gx=gx); hd.fft_conv_accgrad(x, gy, gw=gw)

        def square():
            hd.fft_conv_fprop_tiled(x, wt, n, y=y); hd.fft_conv_bprop_tiled(gy, wt, h, w, n, gx=gx)
            hd.fft_conv_accgrad_tiled(x, gy, n, gw=gw)
        out[f"S{S}_f{f}_fo{fo}_{h}x{w}_k{kh}x{kw}"] = {"basis": f"{nr}x{nc}", "us": timed(rect),
                                                       "square_basis": n, "square_us": timed(square)}
        del x, wt, gy, y, gx, gw
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-passes", action="store_true",
                    help="time the three independent pass calls instead of fprop_save + backward")
    ap.add_argument("--library-basis", action="store_true",
                    help="leave the Fourier basis to the library (28x28 for C2) instead of the one the "
                         "configuration names")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations and the FFT sweep")
    ap.add_argument("--tiled-only", action="store_true",
                    help="only time the tiled layers of the extra block and print them (for profiling runs)")
    ap.add_argument("--rect-only", action="store_true",
                    help="only time the non-square layers of the extra block (rectangular against square "
                         "basis) and print them (for profiling runs)")
    ap.add_argument("--sweep-only", default=None, metavar="SIZES",
                    help="only run the stand-alone FFT sweep at these comma-separated sizes and print it "
                         "(for profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 256 MiB device copy a few times (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (value is one GPU's throughput)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        src = torch.ones(1 << 26, device="cuda", dtype=torch.float32)   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4}))
        return
    import paper_1412_7580_amd as pkg
    from paper_1412_7580_amd import synth

    hd = pkg.Handle(0)
    if args.tiled_only:
        print(json.dumps({"tiled_layers": tiled_layers(hd)}))
        return
    if args.rect_only:
        print(json.dumps({"rectangular_basis": rectangular_layers(hd)}))
        return
    if args.sweep_only:
        sizes = tuple(int(v) for v in args.sweep_only.split(","))
        print(json.dumps({"fft_sweep_256MiB": fft_sweep(hd, sizes=sizes, sizes_1d_only=())}))
        return
    name = args.workload
    cfg = {k: v for k, v in synth.CONV_CONFIGS[name].items() if k != "passes"}
    passes = synth.CONV_CONFIGS[name]["passes"]
    t, host = device_tensors(cfg, synth.CONV_SEEDS[name])

    # The headline runs on the Fourier basis the configuration names (FFT 32x32 for C2); the
    # library's own choice, the smallest basis that holds the image, is timed next to it below.
    basis = None if args.library_basis else cfg["N"]
    if args.library_basis:
        cfg["N"] = library_basis(cfg)
    reuse = (len(passes) == 3) and not args.separate_passes
    if reuse:
        add_saved(hd, t, cfg, basis)
    sec = time_steps(hd, t, cfg, passes, args.steps, args.warmup, reuse, basis)
    flops = direct_flops(cfg) * len(passes)
    value = flops / sec / 1e12

    # Per-kernel durations over a second run of the same region, with per-dispatch events on.
    prof_steps = max(1, min(args.steps, 50))
    kernels = {}
    models = {p: stage_model(cfg, p) for p in passes}

    def entry(ms, model):
        ent = {"ms": round(ms, 5), "GBps": round(model["bytes"] / ms / 1e6, 1)}
        if "flops" in model:
            ent["TFLOPs"] = round(model["flops"] / ms / 1e9, 2)
        return ent

    if reuse:
        km = profile_reuse_step(hd, t, cfg, prof_steps, basis)
        for k, ms in km.items():
            p, s_ = k.split(".")
            if k == "fprop.fft":
                model = models["fprop"]["fft"]
            elif k == "backward.fft":
                model = models["bprop"]["fft_a"]
            elif k == "backward.contraction":
                mb, ma = models["bprop"]["contraction"], models["accgrad"]["contraction"]
                model = {"bytes": mb["bytes"] + ma["bytes"], "flops": mb["flops"] + ma["flops"]}
            elif k == "backward.ifft":
                model = {"bytes": models["bprop"]["ifft"]["bytes"] + models["accgrad"]["ifft"]["bytes"]}
            else:
                model = models[p][s_]
            kernels[k] = entry(ms, model)
            kernels[k]["_model"] = model
    else:
        stage_ms = profile_stages(hd, t, cfg, passes, prof_steps, basis)
        for p in passes:
            for i, s_ in enumerate(STAGES):
                kernels[f"{p}.{s_}"] = entry(stage_ms[p][i], models[p][s_])
                kernels[f"{p}.{s_}"]["_model"] = models[p][s_]
    dom = max(kernels, key=lambda k: kernels[k]["ms"])
    ds = dom.split(".")[1]
    model = kernels[dom]["_model"]
    for k in kernels:
        del kernels[k]["_model"]
    dms = kernels[dom]["ms"]
    if ds == "contraction":
        ach = model["flops"] / dms / 1e9
        kname = "cgemm_pair_kernel" if dom == "backward.contraction" else "cgemm_bins_kernel / cgemm_tail_kernel"
        roof = {"kernel": f"{dom} ({kname})", "bound": "mfma", "achieved": round(ach, 2),
                "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / MFMA_FP32_PEAK_TFLOPS, 4),
                "traffic": None,
                "note": "executed flops: 6 M N K per bin (3-multiplication complex product); "
                        "the 4-multiplication equivalent rate is 4/3 of `achieved`"}
    else:
        ach = model["bytes"] / dms / 1e6
        kn = "fft2d_c2r_kernel" if ds == "ifft" else "fft2d_r2c_kernel"
        roof = {"kernel": f"{dom} ({kn})", "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None}
    tr = MEASURED_TRAFFIC_BYTES.get(name, {}).get(dom) if (reuse or ds == "contraction") else None
    roof["traffic"] = None if tr is None else round(tr)
    roof["algorithmic_bytes"] = model["bytes"]
    roof["avg_launch_ms"] = dms
    roof["launches_averaged"] = prof_steps

    out = {
        "metric": "effective conv TFLOP/s (direct-conv FLOPs), fprop+bprop+accGrad",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{name}: S={cfg['S']} f={cfg['f']} f'={cfg['fo']} input {cfg['h']}x{cfg['w']} "
                               f"kernel {cfg['kh']}x{cfg['kw']} FFT {cfg['N']}x{cfg['N']}, passes " + "+".join(passes),
                   "seed": synth.CONV_SEEDS[name],
                   "calls": "fft_conv_fprop_save + fft_conv_backward (x, w, gy transformed once each)" if reuse
                            else "fft_conv_fprop, fft_conv_bprop, fft_conv_accgrad (independent passes)"},
        "roofline": roof,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, host)
    if not args.no_extra:
        extra = {}
        def measure(c, ps, b, n):
            """Separate passes and, for three-pass workloads, the reuse step of configuration c on
            basis b (None: the library's choice)."""
            s3 = time_steps(hd, t, c, ps, n, 5, False, b)
            sm = profile_stages(hd, t, c, ps, 5, b)
            ent = {"basis": library_basis(c) if b is None else b,
                   "ms_per_step_separate_passes": round(s3 * 1e3, 4),
                   "effective_TFLOPs_separate_passes": round(direct_flops(c) * len(ps) / s3 / 1e12, 2),
                   "kernel_ms[fft,contraction,ifft]": {p: [round(v, 4) for v in sm[p]] for p in ps}}
            if len(ps) == 3:
                add_saved(hd, t, c, b)
                s2 = time_steps(hd, t, c, ps, n, 5, True, b)
                ent["ms_per_step"] = round(s2 * 1e3, 4)
                ent["effective_TFLOPs"] = round(direct_flops(c) * 3 / s2 / 1e12, 2)
            return ent

        if reuse:
            s3 = time_steps(hd, t, cfg, passes, max(10, args.steps // 4), 5, False, basis)
            extra[name + "_separate_passes"] = {"ms_per_step": round(s3 * 1e3, 5),
                                                "effective_TFLOPs": round(flops / s3 / 1e12, 2)}
        if basis is not None and library_basis(cfg) != basis:
            # the same workload with the basis left to the library (Section 3.4's basis search)
            extra[name + "_library_basis"] = measure(cfg, passes, None, max(10, args.steps // 2))
        for other in ("C1", "C3", "C4"):
            if other == name:
                continue
            del t
            torch.cuda.empty_cache()
            ocfg = {k: v for k, v in synth.CONV_CONFIGS[other].items() if k != "passes"}
            opasses = synth.CONV_CONFIGS[other]["passes"]
            t, _ = device_tensors(ocfg, synth.CONV_SEEDS[other])
            n = 20 if other == "C4" else 50
            extra[other] = measure(ocfg, opasses, ocfg["N"], n)
            if library_basis(ocfg) != ocfg["N"]:
                extra[other + "_library_basis"] = measure(ocfg, opasses, None, n)
        del t
        torch.cuda.empty_cache()
        extra["C1_fprop_hip_graph"] = graph_replay_c1(hd)
        extra["tiled_layers"] = tiled_layers(hd)
        torch.cuda.empty_cache()
        extra["paper_table4_layers"] = table4_layers(hd)
        torch.cuda.empty_cache()
        extra["weights_transformed_ahead"] = weights_ahead(hd)
        torch.cuda.empty_cache()
        extra["paper_section5_conv_sweep_3x3"] = conv_sweep_3x3(hd)
        torch.cuda.empty_cache()
        extra["rectangular_basis"] = rectangular_layers(hd)
        torch.cuda.empty_cache()
        extra["device_copy_GBps"] = device_copy_bandwidth()
        torch.cuda.empty_cache()
        extra["fft_sweep_256MiB"] = fft_sweep(hd)
        torch.cuda.empty_cache()
        # the sizes with an odd factor (not part of the benchmark definition's sweep)
        extra["fft_sweep_mixed_sizes_256MiB"] = fft_sweep(hd, sizes=(10, 12, 14, 18, 20, 24, 28, 36, 40, 48, 56, 80, 96, 112),
                                                          sizes_1d_only=(160, 192, 224))
        out["extra"] = extra
    print(json.dumps(out))


if __name__ == "__main__":
    main()
