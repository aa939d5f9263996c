#!/usr/bin/env python3
"""Benchmark of the frequency-domain convolution hot path on one MI355X.

One step = fprop + bprop + accGrad of the headline layer, the largest single-GPU configuration
(S=32, f=f'=128, 64x64 input, 31x31 kernel, 64x64 Fourier basis), as the two calls
fft_conv_fprop_save + fft_conv_backward (x, w and gy are transformed once each).  Inputs are
seeded synthetic fp32 tensors already resident in device memory.  Every step is timed by its own
pair of HIP events; `ms_per_step` is the median.

Prints ONE JSON line: effective TFLOP/s (direct-convolution FLOP count over measured time); a
`roofline` object for the dominant kernel (durations from HIP events that the library attaches
to each dispatch on its own stream) that also holds every kernel of the step (`stages`), the
other three convolution configurations (`other_configs`) and the stand-alone FFT sweep
(`fft_sweep`: GB/s and fraction of 8 TB/s at the ten points of the fifth configuration); and
the fp64 CPU oracle timed on a bounded sample.
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
# and the tables are in profiles/c2_hbm_traffic.md and profiles/c4_hbm_traffic.md.  Keyed by
# workload, then by the stage names of `roofline.stages` (fprop_save + backward step).
MEASURED_TRAFFIC_BYTES = {
    "C2": {
        "fprop.fft": (1.205e4 * 2.0 + 5.225e4) * 1024,
        "fprop.contraction": (2.625e4 * 2.0 + 3.483e4) * 1024,
        "fprop.ifft": (1.748e4 * 2.0 + 1.693e4) * 1024,
        "backward.fft": (8.621e3 * 2.0 + 3.485e4) * 1024,
        "backward.contraction": (5.575e4 * 2.0 + 5.310e4) * 1024,
        "backward.ifft": (2.619e4 * 2.0 + 2.373e4) * 1024,
    },
    "C4": {
        "fprop.fft_a": (3.294e4 * 2.0 + 6.889e4) * 1024,
        "fprop.fft_b": (3.119e4 * 2.0 + 2.823e5) * 1024,
        "fprop.contraction": (1.702e5 * 2.0 + 6.758e4) * 1024,
        "fprop.ifft": (3.388e4 * 2.0 + 1.850e4) * 1024,
        "backward.fft": (9.515e3 * 2.0 + 7.152e4) * 1024,
        "bprop.contraction": (1.692e5 * 2.0 + 6.758e4) * 1024,
        "bprop.ifft": (3.389e4 * 2.0 + 6.554e4) * 1024,
        "accgrad.contraction": (6.763e4 * 2.0 + 2.703e5) * 1024,
        "accgrad.ifft": (1.353e5 * 2.0 + 6.157e4) * 1024,
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
    # accGrad: the three launches (the layer's basis named through the tiled call, which never takes the
    # one-launch kernel) against the one-launch kernel, on this layer (where the ordinary call keeps
    # its three launches) and on one of few samples (where it takes the one launch by itself)
    gw = torch.empty_like(t["w"])
    n = hd.layer_basis(cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])[0]
    acc3 = timed(lambda: hd.fft_conv_accgrad_tiled(t["x"], gy, n, gw=gw))
    acc1 = timed(lambda: hd.fft_conv_accgrad_fused(t["x"], gy, gw=gw))
    xs = torch.empty((2, 64, 13, 13), device="cuda").uniform_(-1, 1)
    gys = torch.empty((2, 64, 11, 11), device="cuda").uniform_(-1, 1)
    gws = torch.empty((64, 64, 3, 3), device="cuda")
    few3 = timed(lambda: hd.fft_conv_accgrad_tiled(xs, gys, n, gw=gws))
    few1 = timed(lambda: hd.fft_conv_accgrad(xs, gys, gw=gws))
    return {"eager_us_per_fprop": round(eager * 1e6, 2), "graph_replay_us_per_fprop": round(replay * 1e6, 2),
            "fused_one_launch_us_per_fprop": round(fused * 1e6, 2),
            "eager_us_per_bprop": round(bprop * 1e6, 2), "fused_one_launch_us_per_bprop": round(bfused * 1e6, 2),
            "three_launch_us_per_accgrad": round(acc3 * 1e6, 2), "fused_one_launch_us_per_accgrad": round(acc1 * 1e6, 2),
            "S2_f64_13x13_three_launch_us_per_accgrad": round(few3 * 1e6, 2),
            "S2_f64_13x13_ordinary_call_us_per_accgrad": round(few1 * 1e6, 2)}


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


def cpu_fft_baseline(n=64, count=4096):
    """The DFT oracle (the definition, O(n^2) per line, fp64, OpenMP over planes) on the first
    `count` planes of the sweep's 2-D input at size n: algorithmic GB/s as for the GPU sweep."""
    import oracle
    from paper_1412_7580_amd import synth
    x = synth.fft_sweep_input(2, n, 0, count)
    t0 = time.perf_counter()
    oracle.dft_r2c_2d(x, n)
    dt = max(time.perf_counter() - t0, 1e-6)
    nbytes = count * (4 * (n - 3) ** 2 + 8 * n * (n // 2 + 1))
    return {"value": round(nbytes / dt / 1e9, 4), "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 DFT by definition, 2-D R2C n={n}: first {count} of the sweep's planes in {dt:.2f}s"}


def device_copy_bandwidth(reps=20, sizes_mib=(256, 1024)):
    """Plain device-to-device copy of 256 MiB and 1 GiB (read + write bytes over time): what the
    memory system delivers to the simplest kernel, for reading the FFT stages' GB/s against."""
    import torch
    out = {}
    for mib in sizes_mib:
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


# ------------------------------------------------------------------ timing and rooflines
def time_steps_events(hd, t, cfg, passes, steps, warmup, reuse=False, basis=None):
    """`warmup` untimed steps, then `steps` steps, each between its own pair of HIP events on the
    stream the library launches on (torch's current stream, which the handle follows), the whole
    region bracketed by synchronize().  Returns (median ms per step over the event pairs, mean ms
    per step by the host clock around the region, [min, max] of the event times)."""
    import statistics
    import torch
    for _ in range(warmup):
        run_step(hd, t, cfg, passes, reuse, basis)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        run_step(hd, t, cfg, passes, reuse, basis)
        b.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps * 1e3
    ms = [a.elapsed_time(b) for a, b in ev]
    return statistics.median(ms), wall, [min(ms), max(ms)]


def profile_kernels(hd, t, cfg, passes, steps, reuse=False, basis=None):
    """Average execution time (ms) of every kernel of one step over `steps` repetitions, from the
    start/stop events the library attaches to each dispatch on its own stream; kernels are named
    by the call they belong to and the label the library reports for them.
    Returns {name: ms} in launch order."""
    import torch
    hd.set_profiling(True)
    acc = {}
    dims = (cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])

    def collect(prefix, backward=False):
        ms, labels = hd.last_kernel_ms(), hd.last_kernel_labels()
        seen = {}
        for v, lab in zip(ms, labels):
            if backward:
                # fft_conv_backward: gy's transform, then the products of bprop and accGrad, in that
                # order when they are separate launches
                n = seen.get(lab, 0); seen[lab] = n + 1
                if lab.startswith("fft"):
                    name = "backward.fft" if lab == "fft.a" else "backward." + lab.replace(".", "_")
                elif lab.endswith(".pair"):
                    name = "backward." + lab.split(".")[0]
                else:
                    name = ("bprop." if n == 0 else "accgrad.") + lab
            else:
                name = prefix + "." + {"fft.ab": "fft", "fft.a": "fft_a", "fft.b": "fft_b"}.get(lab, lab)
            acc[name] = acc.get(name, 0.0) + v

    for _ in range(steps):
        if reuse and len(passes) == 3:
            if basis is None:
                hd.fft_conv_fprop_save(t["x"], t["w"], t["saved"], y=t["y"])
            else:
                hd.fft_conv_fprop_save_tiled(t["x"], t["w"], basis, t["saved"], y=t["y"])
            collect("fprop")
            if basis is None:
                hd.fft_conv_backward(t["gy"], t["saved"], *dims, gx=t["gx"], gw=t["gw"])
            else:
                hd.fft_conv_backward_tiled(t["gy"], t["saved"], *dims, basis, gx=t["gx"], gw=t["gw"])
            collect("backward", backward=True)
        else:
            for p in passes:
                run_step(hd, t, cfg, (p,), False, basis)
                collect(p)
    hd.set_profiling(False)
    torch.cuda.synchronize()
    return {k: v / steps for k, v in acc.items()}


def kernel_model(cfg, name):
    """Algorithmic bytes and executed flops of the kernel called `name` (see profile_kernels)."""
    p, st = name.split(".")
    if p == "backward":
        mb, ma = stage_model(cfg, "bprop"), stage_model(cfg, "accgrad")
        if st == "fft":
            return mb["fft_a"]                      # gy, transformed once for both passes
        if st == "contraction":
            # GYF is an operand of both problems: counted once (the launch can read it once)
            gyf = 8 * cfg["N"] * (cfg["N"] // 2 + 1) * cfg["S"] * cfg["fo"]
            return {"bytes": mb["contraction"]["bytes"] + ma["contraction"]["bytes"] - gyf,
                    "flops": mb["contraction"]["flops"] + ma["contraction"]["flops"]}
        if st == "ifft":
            return {"bytes": mb["ifft"]["bytes"] + ma["ifft"]["bytes"]}
        return mb["fft_a"]                          # tiled layers: gy cut a second time
    return stage_model(cfg, p)[st]


def roofline_entry(ms, model):
    """Roofline of one kernel: the bound is the roofline that allows the least (HBM for the
    transforms; for a contraction whichever of executed flops / 157.3 TFLOP/s and algorithmic
    bytes / 8 TB/s takes longer); frac = that least time over the measured time."""
    ent = {"ms": round(ms, 5), "GBps": round(model["bytes"] / ms / 1e6, 1),
           "frac_hbm": round(model["bytes"] / ms / 1e6 / HBM_PEAK_GBS, 4)}
    t_hbm = model["bytes"] / (HBM_PEAK_GBS * 1e9)
    bound = "hbm"
    if "flops" in model:
        ent["TFLOPs"] = round(model["flops"] / ms / 1e9, 2)
        ent["frac_mfma"] = round(model["flops"] / ms / 1e9 / MFMA_FP32_PEAK_TFLOPS, 4)
        if model["flops"] / (MFMA_FP32_PEAK_TFLOPS * 1e12) > t_hbm:
            bound = "mfma"
    ent["bound"] = bound
    ent["frac"] = ent["frac_mfma"] if bound == "mfma" else ent["frac_hbm"]
    return ent


KERNEL_FUNCTIONS = {   # which kernel function runs a stage (for matching rocprofv3 kernel stats)
    "fft": "fft2d_r2c_multi_kernel (both operands in one launch)", "fft_a": "fft2d_r2c_kernel",
    "fft_b": "fft2d_r2c_kernel", "ifft": "fft2d_c2r_kernel / fft2d_c2r_pair_kernel",
    "contraction": "cgemm_bins_kernel / cgemm_tail_kernel / cgemm_pair_kernel / cgemm_bingroup_kernel",
}

# HBM bytes per launch of the headline's kernels from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (KiB per dispatch, scaled by what the same counters read for a plain 256 MiB copy).  Quoted
# constants, not measured by the run that prints them: the profile named here holds the runs.
QUOTED_TRAFFIC = {
    "C2": ("profiles/c2_hbm_traffic.md", MEASURED_TRAFFIC_BYTES["C2"]),
    "C4": ("profiles/c4_hbm_traffic.md", MEASURED_TRAFFIC_BYTES["C4"]),
}


def measure_config(hd, name, steps, warmup, prof_steps, separate=False, library_basis_=False, per_pass=True):
    """Step time (median of per-step event pairs) and per-kernel rooflines of configuration `name`
    on the Fourier basis it names.  Returns (entry dict, cfg, host inputs)."""
    import torch
    from paper_1412_7580_amd import synth
    cfg = {k: v for k, v in synth.CONV_CONFIGS[name].items() if k != "passes"}
    passes = synth.CONV_CONFIGS[name]["passes"]
    t, host = device_tensors(cfg, synth.CONV_SEEDS[name])
    basis = None if library_basis_ else cfg["N"]
    if library_basis_:
        cfg["N"] = library_basis(cfg)
    reuse = (len(passes) == 3) and not separate
    if reuse:
        add_saved(hd, t, cfg, basis)
    med, wall, rng = time_steps_events(hd, t, cfg, passes, steps, warmup, reuse, basis)
    flops = direct_flops(cfg) * len(passes)
    km = profile_kernels(hd, t, cfg, passes, prof_steps, reuse, basis)
    stages = {k: roofline_entry(ms, kernel_model(cfg, k)) for k, ms in km.items()}
    if reuse and not library_basis_:
        for k, v in QUOTED_TRAFFIC.get(name, (None, {}))[1].items():
            if k in stages:
                stages[k]["traffic"] = round(v)     # quoted constant: see QUOTED_TRAFFIC
    dom = max(stages, key=lambda k: stages[k]["ms"])
    ent = {
        "workload": f"{name}: S={cfg['S']} f={cfg['f']} f'={cfg['fo']} input {cfg['h']}x{cfg['w']} "
                    f"kernel {cfg['kh']}x{cfg['kw']} FFT {cfg['N']}x{cfg['N']}, passes " + "+".join(passes),
        "calls": ("fft_conv_fprop_save + fft_conv_backward (x, w, gy transformed once each)" if reuse
                  else "independent passes: " + ", ".join("fft_conv_" + p for p in passes)),
        "ms_per_step": round(med, 5), "ms_per_step_wall_mean": round(wall, 5),
        "ms_per_step_min_max": [round(v, 5) for v in rng], "steps": steps,
        "effective_TFLOPs": round(flops / med / 1e9, 2),
        "launches_per_step": len(km), "kernel_ms_sum": round(sum(km.values()), 5),
        "dominant": dom, "stages": stages,
    }
    if reuse and per_pass:
        # the passes one by one, each an independent call that transforms both of its operands (the
        # per-pass layout of the paper's Table 4): median of 20 event-timed calls after 5
        per = {}
        for p in passes:
            m1, _, _ = time_steps_events(hd, t, cfg, (p,), 20, 5, False, basis)
            per[p] = {"ms": round(m1, 5), "effective_TFLOPs": round(direct_flops(cfg) / m1 / 1e9, 2)}
        ent["per_pass_independent_calls"] = per
    del t
    torch.cuda.empty_cache()
    return ent, cfg, host, passes, flops


def fft_sweep_median(hd, max_bytes=1 << 28, reps=20, warm=3, sizes=None, sizes_1d_only=()):
    """Stand-alone FFT sweep (the fifth configuration): R2C, then C2R with crop back, of signals
    of n - 3 (squared) samples zero-padded to n, input sized to 256 MiB.  Every repetition has
    its own event pair; reported: median ms, algorithmic GB/s and its fraction of 8 TB/s."""
    import statistics
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
            byts = B * (4 * ni ** dim + 8 * nbins)
            res = {"batch": B, "bytes": byts}
            for nm, fn in (("r2c", fwd), ("c2r", inv)):
                for _ in range(warm):
                    fn()
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
                torch.cuda.synchronize()
                for a, b in ev:
                    a.record(); fn(); b.record()
                torch.cuda.synchronize()
                ms = statistics.median(a.elapsed_time(b) for a, b in ev)
                res[nm] = {"ms": round(ms, 4), "GBps": round(byts / ms / 1e6, 1),
                           "frac": round(byts / ms / 1e6 / HBM_PEAK_GBS, 4)}
            out[f"{dim}d_n{n}"] = res
            del x, X, y
            torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4"],
                    help="headline configuration (default: the largest one, the 64x64 / 31x31 layer)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-passes", action="store_true",
                    help="time the three independent pass calls instead of fprop_save + backward")
    ap.add_argument("--library-basis", action="store_true",
                    help="leave the Fourier basis to the library (28x28 for the 27x27 layer) instead of the "
                         "one the configuration names")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the other configurations, the per-pass calls, the device copy and the FFT sweep of the roofline object (profiling runs)")
    ap.add_argument("--extra", action="store_true",
                    help="also time tiled layers, the paper's Table 4 shapes, weights transformed ahead, the 3x3 "
                         "sweep of Section 5.4, rectangular bases, odd-factor FFT sizes (an `extra` object)")
    ap.add_argument("--tiled-only", action="store_true",
                    help="only time the tiled layers of the extra block and print them (for profiling runs)")
    ap.add_argument("--rect-only", action="store_true",
                    help="only time the non-square layers of the extra block (rectangular against square "
                         "basis) and print them (for profiling runs)")
    ap.add_argument("--sweep-only", default=None, metavar="SIZES",
                    help="only run the stand-alone FFT sweep at these comma-separated sizes and print it "
                         "(for profiling runs)")
    ap.add_argument("--sweep-reps", type=int, default=20)
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
        print(json.dumps({"fft_sweep_256MiB": fft_sweep_median(hd, sizes=sizes, reps=args.sweep_reps)}))
        return
    name = args.workload
    prof_steps = max(1, min(args.steps, 50))
    head, cfg, host, passes, flops = measure_config(hd, name, args.steps, args.warmup, prof_steps,
                                                    args.separate_passes, args.library_basis,
                                                    per_pass=not args.no_others)
    stages = head["stages"]
    dom = head["dominant"]
    d = stages[dom]
    model = kernel_model(cfg, dom)
    traffic_src, traffic_tab = QUOTED_TRAFFIC.get(name, (None, {}))
    traffic = traffic_tab.get(dom) if not (args.separate_passes or args.library_basis) else None
    roof = {
        "kernel": f"{dom} ({KERNEL_FUNCTIONS.get(dom.split('.')[1], 'fft2d_r2c_multi_kernel')})",
        "bound": d["bound"],
        "achieved": d["TFLOPs"] if d["bound"] == "mfma" else d["GBps"],
        "peak": MFMA_FP32_PEAK_TFLOPS if d["bound"] == "mfma" else HBM_PEAK_GBS,
        "unit": "TFLOP/s" if d["bound"] == "mfma" else "GB/s",
        "frac": d["frac"],
        "traffic": None if traffic is None else round(traffic),
        "traffic_source": None if traffic is None else
        f"quoted from {traffic_src} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy); not measured in this run",
        "algorithmic_bytes": model["bytes"],
        "avg_launch_ms": d["ms"], "launches_averaged": prof_steps,
        "note": "per-kernel times: HIP event pair attached to each dispatch on the library's stream; "
                "contraction flops are the executed ones, 6 M N K per bin (3-multiplication complex product)",
        "stages": stages,
    }
    if "flops" in model:
        roof["executed_flops"] = model["flops"]
    if "per_pass_independent_calls" in head:
        roof["per_pass_independent_calls"] = head.pop("per_pass_independent_calls")
    if not args.no_others:
        # what a plain device copy of 256 MiB moves on this machine (read + write), and the dominant
        # kernel's rate against it: the nominal 8 TB/s is not what the simplest kernel gets
        copy = device_copy_bandwidth(sizes_mib=(256,))["256MiB"]
        roof["device_copy_GBps"] = copy
        if "GBps" in d:
            roof["frac_of_device_copy"] = round(d["GBps"] / copy, 4)
        others = {}
        for other in ("C1", "C2", "C3", "C4"):
            if other == name:
                continue
            ent, *_ = measure_config(hd, other, 30, 5, 20)
            others[other] = ent
        roof["other_configs"] = others
        roof["fft_sweep"] = fft_sweep_median(hd, reps=args.sweep_reps)

    out = {
        "metric": "effective conv TFLOP/s (direct-conv FLOPs), fprop+bprop+accGrad; FFT GB/s",
        "value": round(flops / head["ms_per_step"] / 1e9, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "seed": synth.CONV_SEEDS[name], "calls": head["calls"],
                   "timing": f"median of {args.steps} per-step HIP event pairs after {args.warmup} warm-up steps, "
                             f"region bracketed by synchronize(); host-clock mean over the same steps "
                             f"{head['ms_per_step_wall_mean']} ms, min/max {head['ms_per_step_min_max']}",
                   "launches_per_step": head["launches_per_step"], "kernel_ms_sum": head["kernel_ms_sum"]},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, host)
        out["cpu_baseline"]["fft_oracle"] = cpu_fft_baseline()
    if args.extra:
        extra = {}
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
        for nm in ("C2", "C3", "C1"):
            ent, *_ = measure_config(hd, nm, 30, 5, 20, library_basis_=True)
            extra[nm + "_library_basis"] = ent
        # the sizes with an odd factor (not part of the benchmark definition's sweep)
        extra["fft_sweep_mixed_sizes_256MiB"] = fft_sweep_median(
            hd, sizes=(10, 12, 14, 18, 20, 24, 28, 36, 40, 48, 56, 80, 96, 112), sizes_1d_only=(160, 192, 224, 256))
        out["extra"] = extra
    print(json.dumps(out))


if __name__ == "__main__":
    main()
