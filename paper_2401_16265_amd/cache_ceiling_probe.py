"""Diagnostic: is the attainable bandwidth set by HBM or by the path in front of it?

    python3 -m paper_2401_16265_amd.cache_ceiling_probe [--sizes-mib 16,32,...] [--reps R]

Runs libco2's plain copy kernel (co2_copy_f32, 8 bytes per element) back to back on
working sets from well inside the 256 MiB Infinity Cache (the memory-side cache in
front of the HBM stacks) to far beyond it, and prints one JSON line per size with
the event-timed rate.  Under `rocprofv3 --kernel-trace --` the per-dispatch
durations of `copy_f32` (grouped by grid size) give the same figure without launch
gaps.  If a working set that stays in the Infinity Cache is copied no faster than
one streamed from HBM, the ceiling that the sweep runs against is the path between
the L2s and the memory side, not the DRAM.  Launch sequencing and timing only.
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as co2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes-mib", default="16,32,64,96,128,192,256,384,512,1024,4096,16384",
                    help="working sets (source + destination together), MiB")
    ap.add_argument("--reps", type=int, default=0, help="copies per size (0: about 32 GiB moved per size)")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    for mib in (int(v) for v in args.sizes_mib.split(",")):
        n = mib * (1 << 20) // 8                        # 4 bytes read + 4 written per element
        src = torch.randn(n, device=dev)
        dst = torch.empty(n, device=dev)
        reps = args.reps or max(20, min(400, (32 << 30) // (mib << 20)))
        for _ in range(5):
            co2.co2_copy_f32(src, dst, n)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            co2.co2_copy_f32(src, dst, n)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        print(json.dumps({"working_set_mib": mib, "elements": n, "copies": reps,
                          "grid_workgroups": (n + 1023) // 1024,
                          "us_per_copy_incl_launch_gap": round(ms * 1e3, 2),
                          "gbps": round(8 * n / ms / 1e6)}), flush=True)
        del src, dst


if __name__ == "__main__":
    main()
