"""Diagnostic: the same fused sweep on several device allocations held at once.

    python3 -m paper_2401_16265_amd.placement_contrast [--n N] [--K K] [--arenas 3] [--reps 2]

After compacting the free device memory, `--arenas` plain allocations are made and
kept together; the flat buffers of one worker are carved out of each, zero-filled,
and the sweep (steady-state form, K worker buffers) is launched on them in the
order 0,1,2,0,1,2,...  One JSON line reports each launch's duration from HIP
events.  Run under `rocprofv3 --pmc <counters> --` the per-dispatch counter rows of
the `fused_sweep` kernel appear in the same order, so memory-side counters of a
fast and a slow allocation of ONE process can be laid side by side.  Launch
sequencing and timing only; all arithmetic is in libco2's kernels.
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as co2
from . import placement as pl


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1_343_868_928)
    ap.add_argument("--K", type=int, default=8)
    ap.add_argument("--arenas", type=int, default=3)
    ap.add_argument("--reps", type=int, default=2)
    ap.add_argument("--gap", type=int, default=pl.PAGE)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    n, K = args.n, args.K
    seg = co2.SegmentTable([0, n], dev)
    ws = torch.empty(co2.workspace_bytes(n, 1, K), dtype=torch.uint8, device=dev)
    lam = torch.empty(1, dtype=torch.float32, device=dev)
    sizes = [4 * n] * (K + 4)
    compacted = pl.compact_device_memory(dev)
    total = pl.arena_bytes(sizes, args.gap)
    arenas, spacers = [], []
    for i in range(args.arenas):
        if i:
            spacers.append(torch.empty(i * (192 << 20), dtype=torch.uint8, device=dev))
        a = torch.empty(total, dtype=torch.uint8, device=dev)
        a.zero_()
        arenas.append(a)
    stream = torch.cuda.current_stream().cuda_stream

    def launch(ai, t, ev=None):
        v = [x.view(torch.float32) for x in pl.carve(arenas[ai], sizes, args.gap)]
        a, m, x, own, peers = v[0], v[1], v[2], v[3:5], v[5:]
        flags = co2.CO2_FLAG_CARRIED_NORMS if t >= 2 else 0
        p = co2.make_params(seg, K, 1.0, 0.95, 0.5, 1.0, 4, t, flags, ev[0] if ev else None,
                            ev[1] if ev else None)
        co2.co2_outer_step(p, x, a, a, m, [own[t % 2]] + peers, own[(t + 1) % 2], None, lam, ws,
                           stream=stream)

    for ai in range(args.arenas):                    # bring every arena to the steady-state form
        for t in (1, 2):
            launch(ai, t)
    torch.cuda.synchronize()
    order, evs = [], []
    for r in range(args.reps):
        for ai in range(args.arenas):
            ev = (co2.HipEvent(), co2.HipEvent())
            launch(ai, 3 + r, ev)
            torch.cuda.synchronize()
            order.append(ai)
            evs.append(ev)
    ms = [b.elapsed_ms(e) for b, e in evs]
    print(json.dumps({"n": n, "K": K, "gap": args.gap, "compacted_gib": round(compacted / 2**30, 1),
                      "warmup_sweeps_per_arena": 2, "timed_order": order,
                      "sweep_ms": [round(v, 4) for v in ms],
                      "algorithmic_gb": (28 + 4 * K) * n / 1e9}))


if __name__ == "__main__":
    main()
