"""Helpers for the rocprofv3 evidence kept under profiles/.

  python -m paper_2311_11822_amd.profiling copy [MiB]
      runs one plain device-to-device copy of a known size (default 1024 MiB read + 1024 MiB
      written); under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` it calibrates what
      those counters read for known HBM traffic.

  python -m paper_2311_11822_amd.profiling summarize DIR [DIR ...]
      prints, per kernel of this library (and the calibration copy), the number of launches,
      the average duration from the dispatch timestamps and the average of every counter
      found in rocprofv3's csv output below each DIR; where the counters are there, also the L2
      hit rate (TCC_HIT / (TCC_HIT + TCC_MISS)) and the shader clock the kernel ran at
      (4 x SQ_WAVE_CYCLES / (1024 waves x duration), printed for the large-tile kernels, which
      keep one 256-thread workgroup on each of the 256 compute units; a lower bound when the last
      round of workgroups does not fill the chip).

  python -m paper_2311_11822_amd.profiling gemm-yardstick
      times the library GEMM (torch.matmul -> hipBLASLt) on the transposed-A products of the
      clip-weighted gradient's layer shapes: what the vendor's own kernels reach on this device
      for the same flops, without per-sample weights.

  python -m paper_2311_11822_amd.profiling bias-rate
      times dp_bias_norm (column sums of g over the T tokens + their squared norm) on one
      layer of each workload's widest output: bytes of g per second.

  python -m paper_2311_11822_amd.profiling fill-rate
      compiles csrc/probe_fill_rate.hip and runs it: bytes per second the compute units can pull
      from L2, from the memory-side cache and from HBM.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys

KEEP = ("dpbk::", "copy", "Copy", "elementwise")


def run_copy(mib: int) -> None:
    import torch
    n = mib * (1 << 20) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {mib} MiB (read {mib} MiB, wrote {mib} MiB)")


def short(name: str) -> str:
    name = name.replace("dpbk::(anonymous namespace)::", "")
    return name.split("(")[0][:70]


def summarize(dirs) -> None:
    for d in dirs:
        for path in sorted(glob.glob(os.path.join(d, "**", "*.csv"), recursive=True)):
            base = os.path.basename(path)
            if base.endswith("counter_collection.csv"):
                vals = collections.defaultdict(lambda: collections.defaultdict(float))
                # counters are reported once per dispatch and counter
                disp = collections.defaultdict(set)
                dur = collections.defaultdict(float)
                for r in csv.DictReader(open(path)):
                    k = short(r["Kernel_Name"])
                    if not any(x in r["Kernel_Name"] for x in KEEP):
                        continue
                    vals[k][r["Counter_Name"]] += float(r["Counter_Value"])
                    if r["Dispatch_Id"] not in disp[k]:
                        disp[k].add(r["Dispatch_Id"])
                        dur[k] += float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
                print(f"# {path}")
                for k in vals:
                    n = len(disp[k])
                    line = ", ".join(f"{c} = {v / n:.6g}" for c, v in sorted(vals[k].items()))
                    extra = ""
                    if "TCC_HIT_sum" in vals[k] and vals[k]["TCC_HIT_sum"] + vals[k]["TCC_MISS_sum"] > 0:
                        extra += f"; L2 hit rate = {vals[k]['TCC_HIT_sum'] / (vals[k]['TCC_HIT_sum'] + vals[k]['TCC_MISS_sum']):.3f}"
                    if "SQ_WAVE_CYCLES" in vals[k] and "big_kernel" in k and vals[k].get("SQ_WAVES", 0) / n >= 1024:
                        extra += f"; shader clock = {4.0 * vals[k]['SQ_WAVE_CYCLES'] / (1024 * dur[k]):.2f} GHz"
                    print(f"{k}: launches = {n}, avg duration = {dur[k] / n / 1e3:.1f} us, per launch: {line}{extra}")
            elif base.endswith("kernel_stats.csv"):
                print(f"# {path}")
                for r in csv.DictReader(open(path)):
                    if any(x in r["Name"] for x in KEEP):
                        print(f"{short(r['Name'])}: calls = {r['Calls']}, avg = {float(r['AverageNs']) / 1e3:.1f} us, "
                              f"total = {float(r['TotalDurationNs']) / 1e6:.3f} ms, share = {r['Percentage']} %")


def gemm_yardstick() -> None:
    import torch
    shapes = {"cfg4 qkv": (8192, 12288, 36864), "cfg4 out": (8192, 12288, 12288), "cfg4 fc": (8192, 12288, 49152),
              "cfg4 proj": (8192, 49152, 12288), "cfg2 fc": (4096, 1280, 5120), "cfg1 fc": (4096, 768, 3072)}
    for name, (K, M, N) in shapes.items():
        a = torch.randn(K, M, device="cuda", dtype=torch.bfloat16)
        g = torch.randn(K, N, device="cuda", dtype=torch.bfloat16) * 0.01
        for _ in range(3):
            out = a.t() @ g
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
        ev[0].record()
        for i in range(10):
            out = a.t() @ g
            ev[i + 1].record()
        torch.cuda.synchronize()
        ms = sum(ev[i].elapsed_time(ev[i + 1]) for i in range(10)) / 10
        print(f"{name}: a^T g with a [{K}, {M}], g [{K}, {N}] bf16: {ms:.3f} ms, {2.0 * K * M * N / ms / 1e9:.0f} TFLOP/s",
              flush=True)
        del a, g, out


def bias_rate() -> None:
    import torch
    from . import binding as dp
    for name, (B, T, p) in {"cfg4 fc": (4, 2048, 49152), "cfg2 fc": (8, 512, 5120), "cfg1 fc": (16, 256, 3072)}.items():
        g = (torch.randn(B, T, p, device="cuda") * 0.01).to(torch.bfloat16)
        colsum = torch.zeros((B, p), dtype=torch.float32, device="cuda")
        sq = torch.zeros(B, dtype=torch.float32, device="cuda")
        for _ in range(3):
            dp.dp_bias_norm(g, dp.DP_BF16, B, T, p, colsum, sq)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            dp.dp_bias_norm(g, dp.DP_BF16, B, T, p, colsum, sq)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 20
        nbytes = 2.0 * B * T * p
        print(f"{name}: g [{B}, {T}, {p}] bf16 = {nbytes / 1e6:.0f} MB: {ms * 1e3:.1f} us, {nbytes / ms / 1e6:.0f} GB/s", flush=True)


def fill_rate() -> None:
    import subprocess
    import tempfile
    here = os.path.dirname(os.path.abspath(__file__))
    exe = os.path.join(tempfile.mkdtemp(), "probe_fill_rate")
    subprocess.run([os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O3", "-std=c++17",
                    "-Wno-unused-value", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    os.path.join(here, "csrc", "probe_fill_rate.hip"), "-o", exe], check=True,
                   stderr=subprocess.DEVNULL)
    subprocess.run([exe], check=True)


def main() -> None:
    if len(sys.argv) >= 2 and sys.argv[1] == "gemm-yardstick":
        gemm_yardstick()
    elif len(sys.argv) >= 2 and sys.argv[1] == "bias-rate":
        bias_rate()
    elif len(sys.argv) >= 2 and sys.argv[1] == "fill-rate":
        fill_rate()
    elif len(sys.argv) >= 2 and sys.argv[1] == "copy":
        run_copy(int(sys.argv[2]) if len(sys.argv) > 2 else 1024)
    elif len(sys.argv) >= 3 and sys.argv[1] == "summarize":
        summarize(sys.argv[2:])
    else:
        sys.exit(__doc__)


if __name__ == "__main__":
    main()
