"""Condense rocprofv3 CSV output (kernel trace, counter collection) into a short text summary.

    python -m paper_2602_11562_amd.profile_summary <rocprofv3 output dir> [more dirs ...]

Per kernel: launches, average / min / max duration from the kernel trace, and the mean of every collected
counter. Used to write the files under profiles/.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys


def _short(name: str) -> str:
    for key in ("sta_mfma_dma_kernel", "sta_mfma_pipe_kernel", "sta_mfma_kernel", "sta_stream_kernel",
                "sta_generic_kernel", "gsta_one_kernel", "gsta_r_kernel", "gsta_pool_kernel", "gsta_out_kernel",
                "gsta_tiled_kernel", "gsta_generic_kernel"):
        if key in name:
            return key
    return name[:70]


def summarize(d: str) -> str:
    out = [f"== {d}"]
    for f in sorted(glob.glob(os.path.join(d, "**", "*kernel_trace.csv"), recursive=True)):
        dur = collections.defaultdict(list)
        for row in csv.DictReader(open(f)):
            dur[_short(row["Kernel_Name"])].append(int(row["End_Timestamp"]) - int(row["Start_Timestamp"]))
        out.append("kernel trace (durations in us):")
        for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
            out.append(f"  {k:44s} n={len(v):5d} avg={sum(v) / len(v) / 1e3:9.2f} min={min(v) / 1e3:9.2f} "
                       f"max={max(v) / 1e3:9.2f} total_ms={sum(v) / 1e6:9.3f}")
    for f in sorted(glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)):
        agg = collections.defaultdict(lambda: collections.defaultdict(list))
        for row in csv.DictReader(open(f)):
            agg[_short(row["Kernel_Name"])][row["Counter_Name"]].append(float(row["Counter_Value"]))
        out.append("counters (mean per dispatch; max shown because the 1 GiB calibration copies share a kernel name "
                   "with small runtime copies):")
        for k, cs in sorted(agg.items()):
            for c, v in sorted(cs.items()):
                out.append(f"  {k:44s} {c:28s} n={len(v):5d} mean={sum(v) / len(v):18.1f} max={max(v):18.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    for d in sys.argv[1:]:
        print(summarize(d))
