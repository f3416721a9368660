#!/usr/bin/env python3
"""Benchmark of the Book-Keeping clipped-gradient path on one MI355X.

One step = the whole hot path over one synthetic micro-batch: per-layer per-sample norms
(ghost or instantiated by the path rule) -> clip factors -> clip-weighted gradients of every
layer -> Gaussian noise on the rank's shard.  Inputs are resident in HBM before timing.

Prints ONE JSON line: samples/s, ms per step, per-stage times, the roofline of the dominant
kernel (the clip-weighted gradient GEMM, measured with events around its launches inside the
timed loop) and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

PEAK_BF16_FLOPS = 2.5e15       # MI355X dense bf16 MFMA
PEAK_HBM_BYTES = 8.0e12


def workload_flops(w):
    BT = w.B * w.T
    grad = sum(2.0 * BT * d * p for d, p in w.layers)
    norm = 0.0
    for d, p in w.layers:
        ghost = 2 * w.T * w.T <= d * p
        norm += 2.0 * w.B * w.T * w.T * (d + p) if ghost else 2.0 * BT * d * p
    return norm, grad


def ghost_flops_executed(w):
    """Flops the large-tile ghost-norm kernel issues (it uses the Gram matrices' symmetry): per
    sample and tile row I of 256 tokens, one 128 x 128 diagonal tile and 256 x 128 tiles for the
    column blocks J > 2I; each over d + p.  Layers on other kernels count with the nominal figure."""
    total = 0.0
    for d, p in w.layers:
        T = w.T
        if 2 * T * T > d * p or T < 96 or d % 64 or p % 64:
            total += 2.0 * w.B * T * T * (d + p) if 2 * T * T <= d * p else 2.0 * w.B * T * d * p
            continue
        nj, ni = -(-T // 128), -(-T // 256)
        for I in range(ni):
            full = nj - 2 * I - 1
            total += w.B * (2.0 * 128 * 128 + full * 2.0 * 256 * 128) * (d + p)
    return total


def cpu_baseline(w, budget_layers):
    """The oracle as it stands on the host cores, on the first `budget_layers` layers of the
    workload (whole path on them: norms, clip factors, gradient, noise on their elements)."""
    from oracle import bk_oracle as o
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    sub = si.Workload(**{**w.__dict__, "layers": w.layers[:budget_layers], "shard_count": 1, "shard_rank": 0})
    layers = [tuple(si.to_f64(x) for x in si.gen_layer(sub, l)) for l in range(sub.L)]
    # repeated until about 10 s of CPU work have been timed (at most 4 passes); dt = mean pass
    reps, total = 0, 0.0
    while reps < 4 and total < 10.0:
        t0 = time.perf_counter()
        o.private_gradient(layers, sub.clip_mode, sub.R, sub.sigma, sub.stability, sub.noise_seed,
                           sub.noise_step, 0, sub.psi)
        total += time.perf_counter() - t0
        reps += 1
    dt = total / reps
    n_sub, g_sub = workload_flops(sub)
    n_all, g_all = workload_flops(w)
    scale = (n_all + g_all) / (n_sub + g_sub)
    return {
        "value": w.B / (dt * scale), "unit": "samples/s", "cores": cores, "kind": "oracle",
        "sample": f"whole path on the first {budget_layers} of {w.L} layers ({reps} passes, {dt:.2f} s each, float64 numpy), "
                  f"scaled by the flop ratio {scale:.2f}",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg1", choices=sorted(si.WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-noise", action="store_true",
                    help="add the noise in a pass of its own (dp_add_noise) instead of in the gradient "
                         "kernels' epilogue (dp_clipped_grad_noise_multi, the faster of the two)")
    ap.add_argument("--clipping", default="all-layer", choices=["all-layer", "layer-wise"],
                    help="all-layer: one clipping group (the metric's setting); layer-wise: one group per "
                         "layer with thresholds R / sqrt(L), noise in a pass of its own")
    ap.add_argument("--dtype", default=None, choices=["bf16", "f16"],
                    help="store a and g of a 16-bit workload in this type instead of the workload's own")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2311_11822_amd import binding as dp
    from paper_2311_11822_amd.pipeline import BkPipeline

    w = si.WORKLOADS[args.workload]
    if args.dtype and w.dtype != si.F32:
        w = dataclasses.replace(w, dtype={"bf16": si.BF16, "f16": si.F16}[args.dtype])
    baseline = None
    if not args.no_cpu_baseline:
        budget = {"cfg0": 1, "cfg1": 48, "cfg2": 16, "cfg3": 4, "cfg4": 1}[w.name]
        baseline = cpu_baseline(w, budget)

    layers = []
    for l in range(w.L):
        a, g = si.gen_layer(w, l)
        view = (lambda x: x.view(np.int16)) if w.dtype == si.BF16 else (lambda x: x)
        layers.append((torch.from_numpy(view(a)).cuda(), torch.from_numpy(view(g)).cuda()))
    pipe = BkPipeline(layers)
    off, cnt = w.noise_range()
    layerwise = args.clipping == "layer-wise"
    fused = not args.separate_noise and not layerwise
    if layerwise:
        pipe.set_groups(list(range(w.L)), [w.R / w.L ** 0.5] * w.L)

    def step(ev=None):
        if ev:
            ev[0].record()
        pipe.norms()
        if ev:
            ev[1].record()
        if layerwise:
            pipe.clip_grouped(w.clip_mode, w.stability)
        else:
            pipe.clip(w.clip_mode, w.R, w.stability)
        if ev:
            ev[2].record()
        if layerwise:
            pipe.grad_grouped()
        elif fused:
            pipe.grad_noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
        else:
            pipe.grad()
        if ev:
            ev[3].record()
        if layerwise:
            pipe.noise_grouped(w.sigma, w.noise_seed, w.noise_step, off, cnt)
        elif not fused:
            pipe.noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
        if ev:
            ev[4].record()

    for _ in range(args.warmup):
        step()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    stage = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(4)] for e in events])   # ms
    ms_norm, ms_clip, ms_grad, ms_noise = stage.mean(axis=0)
    ms_step = elapsed * 1e3 / args.steps
    per_step = stage.sum(axis=1)               # event time of each step, first norm kernel to last kernel
    props = torch.cuda.get_device_properties(0)
    norm_flops, grad_flops = workload_flops(w)
    grad_launches = -(-w.L // 48) if w.dtype != si.F32 else w.L
    grad_tflops = grad_flops / (ms_grad * 1e-3) / 1e12
    # The gradient of one group of up to 48 layers is one launch of clipped_grad_big_kernel plus,
    # when the last round of tiles is nearly empty, one of clipped_grad_tail_kernel for those
    # tiles; "launch" below means that pair, timed together by the events around the stage.
    # HBM-side bytes per launch from the committed rocprofv3 counter runs
    # (profiles/<workload>_all_kernels.md); null when this workload has not been profiled.
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            per = json.load(f)["per_launch"][w.name]
        traffic = sum(per[k]["fetch_bytes"] + per[k]["write_bytes"]
                      for k in ("clipped_grad_big_kernel", "clipped_grad_tail_kernel") if k in per)
    except (OSError, KeyError, ValueError):
        pass
    out = {
        "metric": "clipped-gradient samples/sec",
        "value": w.B / (ms_step * 1e-3),
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} T={w.T} L={w.L} layers, psi={w.psi}",
                   "clip": "automatic" if w.clip_mode == si.CLIP_AUTOMATIC else "standard",
                   "clipping": args.clipping,
                   "R": w.R, "sigma": w.sigma, "noise_elements": cnt,
                   "noise": "in the gradient kernels' epilogue" if fused else "separate pass"},
        "tflops_nominal": (norm_flops + grad_flops) / (ms_step * 1e-3) / 1e12,
        "pct_bf16_peak": 100.0 * (norm_flops + grad_flops) / (ms_step * 1e-3) / PEAK_BF16_FLOPS,
        "stage_ms": {"norms": ms_norm, "clip": ms_clip, "grad": ms_grad, "noise": ms_noise},
        "norm_stage": {"tflops_nominal": norm_flops / (ms_norm * 1e-3) / 1e12,
                       "tflops_executed": ghost_flops_executed(w) / (ms_norm * 1e-3) / 1e12},
        "ms_per_step_events": {"median": float(np.median(per_step)), "min": float(per_step.min())},
        "seeds": {"data": w.data_seed, "noise": w.noise_seed, "noise_step": w.noise_step},
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "clock_mhz": (getattr(props, "clock_rate", 0) or 0) / 1e3 or None,
                   "peak_bf16_tflops_used": PEAK_BF16_FLOPS / 1e12, "peak_hbm_gbps_used": PEAK_HBM_BYTES / 1e9},
        "noise_gbps": None if fused else 8.0 * cnt / (ms_noise * 1e-3) / 1e9,
        "roofline": {"kernel": "clipped_grad_big_kernel (+ clipped_grad_tail_kernel)" if w.dtype != si.F32
                     else "clipped_grad_f32_kernel",
                     "bound": "mfma",
                     "achieved": grad_tflops, "peak": PEAK_BF16_FLOPS / 1e12, "unit": "TFLOP/s",
                     "frac": grad_tflops * 1e12 / PEAK_BF16_FLOPS,
                     "launches_per_step": grad_launches,
                     "avg_launch_ms": ms_grad / grad_launches,
                     "algorithmic_flops_per_launch": grad_flops / grad_launches,
                     "traffic": traffic},
        "cpu_baseline": baseline,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
