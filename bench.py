#!/usr/bin/env python3
"""Benchmark of the Book-Keeping clipped-gradient path on one MI355X.

One step = the whole hot path over one synthetic micro-batch: per-layer per-sample norms
(ghost or instantiated by the path rule) -> clip factors -> clip-weighted gradients of every
layer -> Gaussian noise on the rank's shard.  Inputs are resident in HBM before timing.

Prints ONE JSON line.  The top-level figures are for the workload of record, cfg4 (one GPU's share
of a 12288-wide block at its real shape, the matrix-core-bound configuration): samples/s, ms per
step, per-stage times, the roofline of the dominant kernel (the clip-weighted gradient GEMM,
timed with events around its launches inside the timed loop) and the CPU oracle timed on a bounded
sample of the same workload.  `per_config` holds the same measurements for cfg1, cfg2 and cfg3
taken in the same process, and `noise_pass` the separate noise pass (dp_add_noise) on cfg4's
shard and on cfg2's whole gradient, as bytes moved per second against the HBM peak.
`ms_per_step_without_stage_events` repeats the K timed steps without the four event records per
step that the stage times need (they cost a fifth of a step on the smallest workload).
"""
from __future__ import annotations

import argparse
import dataclasses
import gc
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
NOISE_ALU_PEAK_BLOCKS = 256 * 4 * 64 * 2.4e9 / 690      # Philox4x32-10 + Box-Muller blocks/s the vector ALUs can issue
HEADLINE = "cfg4"


def workload_flops(w):
    """(norm, gradient) flops by the paper's formulas: ghost norm 2 B T^2 (d + p), instantiated
    norm and weighted gradient 2 B T d p each."""
    BT = w.B * w.T
    grad = sum(2.0 * BT * d * p for d, p in w.layers)
    norm = 0.0
    for d, p in w.layers:
        ghost = 2 * w.T * w.T <= d * p
        norm += 2.0 * w.B * w.T * w.T * (d + p) if ghost else 2.0 * BT * d * p
    return norm, grad


def ghost_flops_executed(w):
    """Flops the ghost-norm kernels issue (they use the Gram matrices' symmetry).  Large-tile
    kernel: per sample and tile row I of 256 tokens, one 128 x 128 diagonal tile and 256 x 128
    tiles for the column blocks J > 2I; whole-sample kernel (129 .. 256 tokens): 36 tiles of
    32 x 32; each over d + p.  Layers on other kernels count with the nominal figure."""
    total = 0.0
    for d, p in w.layers:
        T = w.T
        if 2 * T * T > d * p or T < 96 or d % 64 or p % 64:
            total += 2.0 * w.B * T * T * (d + p) if 2 * T * T <= d * p else 2.0 * w.B * T * d * p
            continue
        if 128 < T <= 256:
            # the whole-sample kernel: the 36 tiles of 32 x 32 on or above the diagonal of the
            # 8 x 8 tile grid, minus nothing (tiles past T are computed on zeros)
            total += w.B * 36 * 2.0 * 32 * 32 * (d + p)
            continue
        nj, ni = -(-T // 128), -(-T // 256)
        for I in range(ni):
            full = nj - 2 * I - 1
            total += w.B * (2.0 * 128 * 128 + full * 2.0 * 256 * 128) * (d + p)
    return total


def grad_flops_executed(w):
    """Flops the gradient stage issues: the contraction 2 B T d p per layer, except for layers on
    the instantiated path, whose gradient is the weighted sum of the per-sample gradients kept by
    the norm kernel (2 B d p)."""
    total = 0.0
    for d, p in w.layers:
        kept = w.dtype != si.F32 and 2 * w.T * w.T > d * p
        total += 2.0 * w.B * d * p if kept else 2.0 * w.B * w.T * d * p
    return total


def cpu_baseline(w, layer_ids, n_samples):
    """The oracle as it stands on the host cores, on a bounded sample of the workload: the whole
    path (norms, clip factors, gradient, noise on the same fraction of the elements) on the listed
    layers and the first n_samples samples; the result is scaled to the workload by the flop ratio."""
    from oracle import bk_oracle as o
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    full = dataclasses.replace(w, layers=tuple(w.layers[l] for l in layer_ids))
    sub = dataclasses.replace(full, B=n_samples)
    layers = []
    for l in range(full.L):
        a, g = si.gen_layer(full, l)
        layers.append((si.to_f64(a[:n_samples]), si.to_f64(g[:n_samples])))
    off, cnt = sub.noise_range()
    # repeated until about 10 s of CPU work have been timed (at most 4 passes); dt = mean pass
    reps, total = 0, 0.0
    while reps < 4 and total < 10.0:
        t0 = time.perf_counter()
        o.private_gradient(layers, sub.clip_mode, sub.R, sub.sigma, sub.stability, sub.noise_seed,
                           sub.noise_step, off, cnt)
        total += time.perf_counter() - t0
        reps += 1
    dt = total / reps
    n_sub, g_sub = workload_flops(sub)
    n_all, g_all = workload_flops(w)
    scale = (n_all + g_all) / (n_sub + g_sub)
    return {
        "value": w.B / (dt * scale), "unit": "samples/s", "cores": cores, "kind": "oracle",
        "sample": f"whole path on layer(s) {list(layer_ids)} of {w.L}, {n_samples} of {w.B} samples, noise on "
                  f"{cnt} elements ({reps} passes, {dt:.2f} s each, float64 numpy); extrapolated to the "
                  f"workload by the flop ratio {scale:.2f}",
    }


# oracle sample per workload: (layer indices, samples), sized for 5-15 s per pass
BASELINE_SAMPLE = {"cfg0": ((0,), 4), "cfg1": (tuple(range(48)), 16), "cfg2": (tuple(range(8)), 8),
                   "cfg3": ((0, 1, 2, 3), 2), "cfg4": ((1,), 2)}


def measure(name, args, torch, BkPipeline, noise_pass=False):
    """Times `args.steps` steps of workload `name` after `args.warmup` untimed ones; returns the
    measurements as a dict.  Device memory is released before returning."""
    w = si.WORKLOADS[name]
    if args.dtype and w.dtype != si.F32:
        w = dataclasses.replace(w, dtype={"bf16": si.BF16, "f16": si.F16}[args.dtype])
    layers = []
    for l in range(w.L):
        a, g = si.gen_layer(w, l)
        view = (lambda x: x.view(np.int16)) if w.dtype == si.BF16 else (lambda x: x)
        layers.append((torch.from_numpy(view(a)).cuda(), torch.from_numpy(view(g)).cuda()))
        if args.zero_operands:
            for x in layers[-1]:
                x.zero_()
        del a, g
    pipe = BkPipeline(layers)
    off, cnt = w.noise_range()
    passes = args.clipping == "layer-wise-passes"
    layerwise = args.clipping == "layer-wise"
    fused = not args.separate_noise and not layerwise
    if layerwise or passes:
        pipe.set_groups(list(range(w.L)), [w.R / w.L ** 0.5] * w.L)

    def step(ev=None):
        if ev:
            ev[0].record()
        if passes:
            # norms -> factors -> gradients (+ noise) pass by pass: one call, timed as one stage
            pipe.layerwise_step(w.clip_mode, w.stability, w.sigma, w.noise_seed, w.noise_step, off, cnt,
                                layers_per_pass=args.layers_per_pass)
            if ev:
                for e in ev[1:]:
                    e.record()
            return
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

    # The same K steps once more without the per-stage event records: on the small workloads the
    # four records per step cost more than the launches they separate.
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_plain = (time.perf_counter() - t0) * 1e3 / args.steps

    stage = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(4)] for e in events])   # ms
    ms_norm, ms_clip, ms_grad, ms_noise = stage.mean(axis=0)
    ms_step = elapsed * 1e3 / args.steps
    per_step = stage.sum(axis=1)               # event time of each step, first norm kernel to last kernel
    norm_flops, grad_flops = workload_flops(w)
    norm_exec = ghost_flops_executed(w)
    grad_exec = grad_flops_executed(w)
    kept_bytes = sum(4.0 * (w.B + 1) * d * p for d, p in w.layers if w.dtype != si.F32 and 2 * w.T * w.T > d * p)
    grad_launches = -(-w.L // 48) if w.dtype != si.F32 else w.L
    res = {
        "workload": f"{w.name}: B={w.B} T={w.T} L={w.L} layers, psi={w.psi}",
        "dtype": w.dtype,
        "clip": "automatic" if w.clip_mode == si.CLIP_AUTOMATIC else "standard",
        "noise": "in the gradient kernels' epilogue" if fused else "separate pass",
        "noise_elements": cnt,
        "ms_per_step": ms_step,
        "samples_per_s": w.B / (ms_step * 1e-3),
        "ms_per_step_events": {"median": float(np.median(per_step)), "min": float(per_step.min())},
        "ms_per_step_without_stage_events": ms_plain,
        "samples_per_s_without_stage_events": w.B / (ms_plain * 1e-3),
        "stage_ms": {"norms": float(ms_norm), "clip": float(ms_clip), "grad": float(ms_grad), "noise": float(ms_noise)},
        # executed = what the kernels issue (the ghost-norm kernel skips the lower triangle of the
        # symmetric Gram matrices); model = the paper's operation counts (complexity table, section 3)
        "tflops_executed": (norm_exec + grad_exec) / (ms_step * 1e-3) / 1e12,
        "pct_bf16_peak": 100.0 * (norm_exec + grad_exec) / (ms_step * 1e-3) / PEAK_BF16_FLOPS,
        "tflops_model": (norm_flops + grad_flops) / (ms_step * 1e-3) / 1e12,
        "pct_bf16_peak_model_flops": 100.0 * (norm_flops + grad_flops) / (ms_step * 1e-3) / PEAK_BF16_FLOPS,
        "norm_stage": {"tflops_model": norm_flops / (ms_norm * 1e-3) / 1e12,
                       "tflops_executed": norm_exec / (ms_norm * 1e-3) / 1e12},
        # layers on the instantiated path take their gradient from the kept per-sample gradients
        # (kept_weighted_sum_kernel: B + 1 arrays of d p floats move), the others from the
        # contraction over a and g (clipped_grad_big_kernel)
        "grad_stage": {"tflops": grad_exec / (ms_grad * 1e-3) / 1e12,
                       "frac_bf16_peak": grad_exec / (ms_grad * 1e-3) / PEAK_BF16_FLOPS,
                       "launches_per_step": grad_launches,
                       "flops_per_step": grad_exec,
                       "kept_gradient_bytes": kept_bytes,
                       "kept_gradient_gbps": kept_bytes / (ms_grad * 1e-3) / 1e9 if kept_bytes else None},
    }
    if noise_pass:
        # the separate noise pass on this workload's shard: 4 bytes read + 4 written per element
        for _ in range(2):
            pipe.noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        ev[0].record()
        for k in range(args.steps):
            pipe.noise(w.sigma, w.R, w.noise_seed, w.noise_step + 1 + k, off, cnt)
            ev[k + 1].record()
        torch.cuda.synchronize()
        ms = np.array([ev[k].elapsed_time(ev[k + 1]) for k in range(args.steps)])
        gbps = 8.0 * cnt / (ms.mean() * 1e-3) / 1e9
        res["noise_pass"] = {"kernel": "noise_bulk_kernel", "elements": cnt, "bytes": 8 * cnt,
                             "ms": float(ms.mean()), "ms_min": float(ms.min()),
                             "gbps": gbps, "frac_hbm_peak": gbps * 1e9 / PEAK_HBM_BYTES,
                             # the generator's instruction stream is ~690 vector-ALU clocks per
                             # 4-element block and wave: 256 CUs x 4 SIMDs x 64 lanes x 2.4 GHz / 690
                             "gblocks_per_s": cnt / 4 / (ms.mean() * 1e-3) / 1e9,
                             "frac_alu_peak": cnt / 4 / (ms.mean() * 1e-3) / NOISE_ALU_PEAK_BLOCKS}
    del pipe, layers
    gc.collect()
    torch.cuda.empty_cache()
    return w, res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(si.WORKLOADS),
                    help="workload of the top-level figures (default: cfg4, the metric's configuration)")
    ap.add_argument("--only", action="store_true",
                    help="measure the --workload alone: no per_config block, no cfg2 noise pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-noise", action="store_true",
                    help="add the noise in a pass of its own (dp_add_noise) instead of in the gradient "
                         "kernels' epilogue (dp_clipped_grad_noise_multi, the faster of the two)")
    ap.add_argument("--clipping", default="all-layer", choices=["all-layer", "layer-wise", "layer-wise-passes"],
                    help="all-layer: one clipping group (the metric's setting); layer-wise: one group per "
                         "layer with thresholds R / sqrt(L), all norms then all gradients, noise in a pass of "
                         "its own; layer-wise-passes: the same result without book-keeping "
                         "(dp_layerwise_clipped_grad: norms, factors, gradients and noise pass by pass; the "
                         "stage times then hold the whole step under 'norms')")
    ap.add_argument("--layers-per-pass", type=int, default=0,
                    help="layer-wise-passes: layers per pass (0: the library's own pass size)")
    ap.add_argument("--dtype", default=None, choices=["bf16", "f16"],
                    help="store a and g of a 16-bit workload in this type instead of the workload's own")
    ap.add_argument("--zero-operands", action="store_true",
                    help="diagnostic: all-zero a and g (same kernels, addresses and memory traffic, no bit "
                         "toggling in the matrix cores); the difference to the normal run is the clock the "
                         "device sustains under the power of real data.  Not a valid benchmark figure")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2311_11822_amd.pipeline import BkPipeline

    baseline = None
    if not args.no_cpu_baseline:
        ids, n = BASELINE_SAMPLE[args.workload]
        baseline = cpu_baseline(si.WORKLOADS[args.workload], ids, n)

    w, head = measure(args.workload, args, torch, BkPipeline, noise_pass=True)
    per_config, noise_pass = {}, {f"{w.name}_shard": head.pop("noise_pass")}
    if not args.only:
        for name in ("cfg1", "cfg2", "cfg3"):
            if name == args.workload:
                continue
            _, r = measure(name, args, torch, BkPipeline, noise_pass=(name == "cfg2"))
            if "noise_pass" in r:
                noise_pass[f"{name}_full"] = r.pop("noise_pass")
            per_config[name] = r

    # Bytes per launch that missed the XCDs' L2 caches (rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled
    # by what the same counters read for a device copy of known size; served by the memory-side
    # cache or by HBM): profiles/l2_miss_traffic.json, written from the committed counter runs;
    # null when this workload has not been profiled.
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "l2_miss_traffic.json")) as f:
            per = json.load(f)["per_launch"][w.name]
        traffic = sum(per[k]["fetch_bytes"] + per[k]["write_bytes"]
                      for k in ("clipped_grad_big_kernel", "clipped_grad_tail_kernel") if k in per)
    except (OSError, KeyError, ValueError):
        pass
    props = torch.cuda.get_device_properties(0)
    gs = head["grad_stage"]
    ms_grad = head["stage_ms"]["grad"]
    out = {
        "metric": "clipped-gradient samples/sec",
        "value": head["samples_per_s"],
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic" if not args.zero_operands else "all-zero operands (diagnostic run, not a benchmark figure)",
        "config": {"workload": head["workload"], "clip": head["clip"], "clipping": args.clipping,
                   "R": w.R, "sigma": w.sigma, "noise_elements": head["noise_elements"], "noise": head["noise"]},
        "tflops_executed": head["tflops_executed"],
        "pct_bf16_peak": head["pct_bf16_peak"],
        "tflops_model": head["tflops_model"],
        "pct_bf16_peak_model_flops": head["pct_bf16_peak_model_flops"],
        "stage_ms": head["stage_ms"],
        "norm_stage": head["norm_stage"],
        "ms_per_step_events": head["ms_per_step_events"],
        "ms_per_step_without_stage_events": head["ms_per_step_without_stage_events"],
        "seeds": {"data": w.data_seed, "noise": w.noise_seed, "noise_step": w.noise_step},
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "clock_mhz": (getattr(props, "clock_rate", 0) or 0) / 1e3 or None,
                   "peak_bf16_tflops_used": PEAK_BF16_FLOPS / 1e12, "peak_hbm_gbps_used": PEAK_HBM_BYTES / 1e9},
        # separate noise pass (dp_add_noise) on this workload's shard; the timed step above adds
        # the noise in the gradient kernels' epilogue unless --separate-noise
        "noise_gbps": noise_pass[f"{w.name}_shard"]["gbps"],
        "noise_pass": noise_pass,
        # The gradient of one group of up to 48 layers is one launch of clipped_grad_big_kernel
        # plus, when the last round of tiles is nearly empty, one of clipped_grad_tail_kernel for
        # those tiles; "launch" below means that pair, timed together by the events around the stage.
        "roofline": {"kernel": "clipped_grad_big_kernel (+ clipped_grad_tail_kernel)" if w.dtype != si.F32
                     else "clipped_grad_f32_kernel",
                     "bound": "mfma",
                     "achieved": gs["tflops"], "peak": PEAK_BF16_FLOPS / 1e12, "unit": "TFLOP/s",
                     "frac": gs["frac_bf16_peak"],
                     "launches_per_step": gs["launches_per_step"],
                     "avg_launch_ms": ms_grad / gs["launches_per_step"],
                     "algorithmic_flops_per_launch": gs["flops_per_step"] / gs["launches_per_step"],
                     "traffic": traffic},
        "per_config": per_config,
        "cpu_baseline": baseline,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
