"""Helpers for the rocprofv3 evidence kept under profiles/.

  python -m paper_2311_11822_amd.profiling copy [MiB]
      runs one plain device-to-device copy of a known size (default 1024 MiB read + 1024 MiB
      written); under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` it calibrates what
      those counters read for known HBM traffic.

  python -m paper_2311_11822_amd.profiling summarize DIR [DIR ...]
      prints, per kernel of this library (and the calibration copy), the number of launches,
      the average duration from the dispatch timestamps and the average of every counter
      found in rocprofv3's csv output below each DIR.
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
                    print(f"{k}: launches = {n}, avg duration = {dur[k] / n / 1e3:.1f} us, per launch: {line}")
            elif base.endswith("kernel_stats.csv"):
                print(f"# {path}")
                for r in csv.DictReader(open(path)):
                    if any(x in r["Name"] for x in KEEP):
                        print(f"{short(r['Name'])}: calls = {r['Calls']}, avg = {float(r['AverageNs']) / 1e3:.1f} us, "
                              f"total = {float(r['TotalDurationNs']) / 1e6:.3f} ms, share = {r['Percentage']} %")


def main() -> None:
    if len(sys.argv) >= 2 and sys.argv[1] == "copy":
        run_copy(int(sys.argv[2]) if len(sys.argv) > 2 else 1024)
    elif len(sys.argv) >= 3 and sys.argv[1] == "summarize":
        summarize(sys.argv[2:])
    else:
        sys.exit(__doc__)


if __name__ == "__main__":
    main()
