#!/usr/bin/env python3
"""Benchmark of the CO2 outer update on one MI355X.

A "step" is one pass of the whole outer update (pseudo-gradient, K-way mean,
the two segment norms and Lambda of Eq. 3, momentum, clipping, outer iterate,
writes of params/anchor/momentum/delta_out) over the 1.3B-parameter, K=8
workload, with every buffer already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps 20] [--warmup 3] [--form carried|two_pass]
                  [--workload 1p3b|gpt2s|7b_shard|tiny] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak

# HBM bytes per launch of the fused sweep measured with rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, scaled by the copy-kernel calibration);
# summaries under profiles/.  None until measured for a workload.
MEASURED_TRAFFIC_BYTES = {
    # profiles/fused_sweep_1p3b_k8_hbm_counters.md
    ("1p3b", "f32", 8): 8.0800e10,
    # profiles/fused_sweep_bf16_deltas_1p3b_k8.md: (2 x 18373268 + 18537254) KiB
    ("1p3b", "bf16", 8): 5.6610e10,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--form", choices=["carried", "two_pass"], default="carried",
                    help="carried: steady-state single pass (norm sums carried from the "
                         "previous round's sweep); two_pass: separate norm pass every round")
    ap.add_argument("--workload", default="1p3b")
    ap.add_argument("--K", type=int, default=0, help="override the workload's worker count")
    ap.add_argument("--deltas", choices=["f32", "bf16"], default="f32",
                    help="storage type of the K pseudo-gradient buffers and of delta_out "
                         "(bf16: reduced-precision transport, co2_outer_step_bf16)")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="allocate every buffer on its own instead of carving all of them out of "
                         "one device allocation (the layout the library recommends)")
    ap.add_argument("--placement-candidates", type=int, default=3,
                    help="plain device allocations tried for the buffers after the free device memory "
                         "has been compacted; the sweep is timed on each candidate and the fastest "
                         "layout is kept.  0 = no compaction, no search: the first plain allocation "
                         "as it comes")
    ap.add_argument("--piece-major", action="store_true",
                    help="also try two piece-major buffer sets (co2_buffer_set_create) as candidates")
    ap.add_argument("--hip-graph", action="store_true",
                    help="also capture two consecutive rounds into a HIP graph and time its replays; "
                         "value and ms_per_step then come from the replays (launch-bound small "
                         "workloads), the roofline still from the eager launches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=int, default=160_000_000)
    return ap.parse_args()


def cpu_baseline(cfg, table, sample_elems: int, gen_device="cpu"):
    """The oracle, as it stands, single-threaded on this host, on a bounded sample
    of whole segments of the same workload (same K, same drift recipe)."""
    import numpy as np
    import torch

    import co2_inputs
    from oracle import co2_oracle

    # whole segments, largest-first skipped if too big, until the budget is filled
    sizes = [table[s + 1] - table[s] for s in range(len(table) - 1)]
    chosen, total = [], 0
    for s in range(len(sizes) - 1, -1, -1):          # from the last layers backwards
        if total + sizes[s] <= sample_elems:
            chosen.append(s)
            total += sizes[s]
    chosen.sort()
    otable = np.concatenate([[0], np.cumsum([sizes[s] for s in chosen])]).astype(np.int64)
    n = int(otable[-1])

    def draw(std, bid, student=False):
        # drawn on the GPU when there is one (the Student-t recipe is slow on the
        # host), then handed to the oracle as host arrays
        t = torch.empty(n, dtype=torch.float32, device=gen_device)
        if student:
            co2_inputs.fill_student_t_(t, std, cfg.drift_nu, co2_inputs.seed_for(cfg.seed, bid))
        else:
            co2_inputs.fill_normal_(t, std, co2_inputs.seed_for(cfg.seed, bid))
        return t.cpu().numpy()

    st = cfg.drift == "student_t"
    a = draw(cfg.param_std, 1)
    m = draw(cfg.momentum_std, 2)
    x = a + draw(cfg.drift_scale, 100, st)
    d = [draw(cfg.drift_scale, 200 + k, st) for k in range(cfg.K)]
    kw = dict(seg_off=otable, alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau)
    co2_oracle.outer_step_f32(x=x, a=a, m=m, deltas=d, step=1, **kw)      # warm the pages
    reps, t0 = 0, time.perf_counter()
    while True:
        co2_oracle.outer_step_f32(x=x, a=a, m=m, deltas=d, step=2 + reps, **kw)
        reps += 1
        el = time.perf_counter() - t0
        if el > 12.0 or reps >= 64:
            break
    return {"value": n * reps / el, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(chosen)} whole segments ({n} of {table[-1]} params) of the same "
                      f"workload, K={cfg.K}, {reps} outer steps in {el:.1f} s, g++ -O2, 1 thread"}


def overlap_bench(args):
    """Overlapped-round workload: tau fused AdamW steps on the main stream while the
    outer update (split form) runs on a side stream; steady-state round time against
    the same launches issued serially.  Prints its own JSON line."""
    import statistics

    import torch

    import co2_inputs
    import paper_2401_16265_amd as co2
    from paper_2401_16265_amd.schedule import AdamWConfig, CO2Worker

    from paper_2401_16265_amd.placement import compact_device_memory

    dev = torch.device("cuda:0")
    compacted = compact_device_memory(dev)       # same starting point whatever ran on the device before
    cfg = co2_inputs.CONFIGS["350m_overlap"]
    table = co2_inputs.config_table(cfg)
    seg = co2.SegmentTable(table, dev)
    n, K, tau = seg.n, cfg.K, cfg.tau
    hp = {k: v for k, v in cfg.adamw.items() if k != "grad_std"}
    init = co2_inputs.fill_normal_(torch.empty(n, dtype=torch.float32, device=dev), cfg.param_std,
                                   co2_inputs.seed_for(cfg.seed, 1))
    grads = [co2_inputs.fill_bf16_normal_(torch.empty(n, dtype=torch.bfloat16, device=dev),
                                          cfg.adamw["grad_std"], co2_inputs.seed_for(cfg.seed, 10 + k))
             for k in range(tau)]
    rounds = max(args.steps, 12)
    res = {}
    for mode in ("serial", "overlapped"):
        w = CO2Worker(seg, K, tau, cfg.alpha, cfg.beta, cfg.phi, cfg.c, AdamWConfig(**hp), dev, init)
        for j, pb in enumerate(w.peers):
            co2_inputs.fill_normal_(pb, cfg.drift_scale, co2_inputs.seed_for(cfg.seed, 200 + j))
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(rounds + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(rounds):
            evs[r].record()
            (w.round_overlapped if mode == "overlapped" else w.round_serial)(grads)
        evs[rounds].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per = [evs[r].elapsed_time(evs[r + 1]) for r in range(rounds)]
        res[mode] = {"median_ms": statistics.median(per[10:]), "min_ms": min(per[10:]),
                     "wall_ms_per_round": wall * 1e3 / rounds}
        del w
        torch.cuda.empty_cache()
    bytes_round = (26 * tau + 8 + 4) * n + (16 + 4 * K) * n   # AdamW steps (+dout, +anchor read) + split outer update
    out = {"metric": "overlapped round time (tau AdamW steps + outer update)",
           "value": res["overlapped"]["median_ms"], "unit": "ms", "n_gpus": 1, "steps": rounds,
           "warmup": 10, "ms_per_step": res["overlapped"]["median_ms"], "higher_is_better": False,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{cfg.name}: n={n}, K={K}, tau={tau}, bf16 grads, fp32 master",
                      "compacted_gib": round(compacted / 2**30, 1)},
           "serial": res["serial"], "overlapped": res["overlapped"],
           "overlap_speedup": res["serial"]["median_ms"] / res["overlapped"]["median_ms"],
           "round_gbps_algorithmic": bytes_round / (res["overlapped"]["median_ms"] * 1e-3) / 1e9}
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the K workers are K device buffers "
              "reduced in-kernel); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import co2_inputs
    import paper_2401_16265_amd as co2

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.workload == "350m_overlap":
        return overlap_bench(args)
    dev = torch.device("cuda:0")
    cfg = co2_inputs.CONFIGS[args.workload]
    if args.K:
        import dataclasses
        cfg = dataclasses.replace(cfg, K=args.K)
    table = co2_inputs.config_table(cfg)
    seg = co2.SegmentTable(table, dev)
    n, S, K = seg.n, seg.S, cfg.K
    f32 = dict(dtype=torch.float32, device=dev)

    # ---- resident state: params, anchor, momentum, K-1 peers, 2 own (ping-pong).
    # All flat buffers are carved out of ONE device allocation.  The sweep streams
    # 3+K+1 buffers in lock step and its duration depends on where they lie relative
    # to each other in HBM (up to 10 % between allocations, 3 % between gaps), so the
    # allocation and the gap are chosen by timing the sweep itself on a few candidates
    # before anything is initialised (paper_2401_16265_amd/placement.py).
    bf16 = args.deltas == "bf16"
    dd = dict(dtype=torch.bfloat16 if bf16 else torch.float32, device=dev)
    lam = torch.empty(S, **f32)
    ws = torch.empty(co2.workspace_bytes(n, S, K), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    carried = args.form == "carried"
    entry = co2.co2_outer_step_bf16 if bf16 else co2.co2_outer_step

    def typed(views):
        a, m, x = (v.view(torch.float32) for v in views[:3])
        ds = [v.view(dd["dtype"]) for v in views[3:]]
        return a, m, x, ds[:2], ds[2:]

    def launch(bufs, t, ev=None, clipped=None, on=None):
        """One outer step of round t on stream `on` (default: the current stream)."""
        a, m, x, own, peers = bufs
        cur, nxt = own[t % 2], own[(t + 1) % 2]          # deltas[0] = last round's delta_out
        flags = co2.CO2_FLAG_CARRIED_NORMS if (carried and t >= 2) else 0
        p = co2.make_params(seg, K, cfg.alpha, cfg.beta, cfg.phi, cfg.c, cfg.tau, t, flags,
                            ev[0] if ev else None, ev[1] if ev else None, clipped)
        entry(p, x, a, a, m, [cur] + peers, nxt, None, lam, ws, stream=on or stream)

    def probe(views, reps=3):
        """Median duration (ms) of the sweep kernel over `reps` launches on these buffers."""
        bufs = typed(views)
        evs = [(co2.HipEvent(), co2.HipEvent()) for _ in range(reps)]
        for t in range(1, 3):
            launch(bufs, t)
        for i in range(reps):
            launch(bufs, 3 + i, evs[i])
        torch.cuda.synchronize()
        return sorted(b.elapsed_ms(e) for b, e in evs)[reps // 2]

    placement = None
    if args.separate_allocations:
        a = torch.empty(n, **f32); m = torch.empty(n, **f32); x = torch.empty(n, **f32)
        own = [torch.empty(n, **dd), torch.empty(n, **dd)]
        peers = [torch.empty(n, **dd) for _ in range(K - 1)]
    else:
        from paper_2401_16265_amd import placement as pl
        dbytes = n * (2 if bf16 else 4)
        sizes = [4 * n] * 3 + [dbytes] * (K + 1)
        search = args.placement_candidates > 0
        placement = pl.choose_placement(sizes, probe if search else None, dev,
                                        candidates=args.placement_candidates,
                                        pieces=pl.DEFAULT_PIECES if args.piece_major else (),
                                        gaps=pl.DEFAULT_GAPS if search else (pl.PAGE,))
        a, m, x, own, peers = typed(placement.views)
    student = cfg.drift == "student_t"

    def drift(t, bid):
        sd = co2_inputs.seed_for(cfg.seed, bid)
        dst = x if t.dtype == torch.bfloat16 else t       # x doubles as fp32 scratch here
        if student:
            co2_inputs.fill_student_t_(dst, cfg.drift_scale, cfg.drift_nu, sd)
        else:
            co2_inputs.fill_normal_(dst, cfg.drift_scale, sd)
        if dst is not t:
            t.copy_(dst)

    co2_inputs.fill_normal_(a, cfg.param_std, co2_inputs.seed_for(cfg.seed, 1))
    co2_inputs.fill_normal_(m, cfg.momentum_std, co2_inputs.seed_for(cfg.seed, 2))
    drift(own[1], 99)
    for k, pb in enumerate(peers):
        drift(pb, 200 + k)
    drift(x, 100); x.add_(a)                                # local params = anchor + drift
    torch.cuda.synchronize()

    step_no = [1]
    bufs = (a, m, x, own, peers)

    def one_step(ev=None):
        launch(bufs, step_no[0], ev)
        step_no[0] += 1

    warmup = max(args.warmup, 2 if carried else 0)   # carried sums exist from round 2 on
    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()

    events = [(co2.HipEvent(), co2.HipEvent()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed * 1e3 / args.steps
    launch_mode = "eager"
    if args.hip_graph:
        # two rounds = one period of the delta_out ping-pong; step parity continues from the eager loop
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        t_cap = step_no[0] + (step_no[0] % 2)               # even round first
        with torch.cuda.graph(graph, stream=side):
            capturing = torch.cuda.current_stream().cuda_stream
            launch(bufs, t_cap, on=capturing)
            launch(bufs, t_cap + 1, on=capturing)
        if step_no[0] % 2:
            one_step()                                      # bring the ping-pong to an even round
        replays = max(1, args.steps // 2)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / (2 * replays)
        launch_mode = f"hip graph of 2 rounds, {replays} replays (eager: {elapsed * 1e3 / args.steps:.4f} ms/step)"
        del graph
    sweep_ms = sum(b.elapsed_ms(e) for b, e in events) / args.steps
    per_elem = (26 + 2 * K) if bf16 else (28 + 4 * K)   # algorithmic bytes per coordinate, one sweep
    sweep_bytes = per_elem * n
    achieved = sweep_bytes / (sweep_ms * 1e-3) / 1e9

    # ---- one more step, untimed, that also counts the coordinates the clip changed
    clipped = torch.zeros(S, dtype=torch.int64, device=dev)
    launch(bufs, step_no[0], None, clipped)
    step_no[0] += 1
    torch.cuda.synchronize()
    clipped_count = int(clipped.sum().item())

    # ---- yardstick: plain copy kernel over one buffer pair (8 B/element)
    cb, ce = co2.HipEvent(), co2.HipEvent()
    co2.co2_copy_f32(a, x, n, stream=stream)
    cb.record(stream)
    for _ in range(5):
        co2.co2_copy_f32(a, x, n, stream=stream)
    ce.record(stream)
    ce.synchronize()
    copy_gbps = 8 * n * 5 / (cb.elapsed_ms(ce) * 1e-3) / 1e9

    out = {
        "metric": "outer-step params/sec",
        "value": n / (ms_per_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={n} fp32 params, S={S} segments, K={K} worker "
                               f"buffers, {cfg.drift} drift, beta={cfg.beta} phi={cfg.phi} "
                               f"c={cfg.c}", "form": args.form, "deltas": args.deltas, "launch": launch_mode,
                   "placement": ("separate allocations" if placement is None else
                                 placement.report() if args.placement_candidates > 0 else
                                 "first allocation"),
                   "clipped_coordinates_in_one_step": clipped_count,
                   "step_gbps_algorithmic": (per_elem + (0 if carried else (6 if bf16 else 8))) * n
                                            / (ms_per_step * 1e-3) / 1e9},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, args.deltas, K)),   # the sweep's, either form
                     "kernel": "fused_sweep", "kernel_ms": sweep_ms,
                     "algorithmic_bytes": sweep_bytes, "copy_kernel_gbps": copy_gbps},
    }
    del a, m, x, own, peers, bufs
    torch.cuda.synchronize()
    if placement is not None:
        placement.release()
    del placement
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline and not bf16:
        out["cpu_baseline"] = cpu_baseline(cfg, table, args.cpu_sample_elems, dev)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
