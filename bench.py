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
    ("1p3b", "f32", 8): (8.0800e10, "profiles/fused_sweep_1p3b_k8_hbm_counters.md (profiled constant, "
                                    "not measured in this run)"),
    # (2 x 18373268 + 18537254) KiB
    ("1p3b", "bf16", 8): (5.6610e10, "profiles/fused_sweep_bf16_deltas_1p3b_k8.md (profiled constant, "
                                     "not measured in this run)"),
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
    ap.add_argument("--deltas", choices=["f32", "bf16", "f16"], default="f32",
                    help="storage type of the K pseudo-gradient buffers and of delta_out "
                         "(bf16: reduced-precision transport, co2_outer_step_bf16)")
    ap.add_argument("--layout", choices=["piece-major", "search", "first", "separate"], default="piece-major",
                    help="where the flat buffers live.  piece-major (default): one co2_buffer_set with "
                         "64 MiB pieces, made after the free device memory has been compacted; no "
                         "selection by timing (a plain first allocation is timed beforehand only to be "
                         "reported).  search: compaction, then the sweep is timed on "
                         "--placement-candidates plain allocations x three gaps (plus buffer sets of the "
                         "--piece-mib sizes) and the fastest layout is kept.  first: one plain allocation "
                         "as the device hands it out.  separate: one allocation per buffer")
    ap.add_argument("--placement-candidates", type=int, default=3,
                    help="--layout search: plain device allocations tried")
    ap.add_argument("--piece-mib", default="",
                    help="comma-separated piece sizes in MiB of the buffer sets (piece-major: the first "
                         "one, default 64; search: all of them as extra candidates, default none)")
    ap.add_argument("--hip-graph", action="store_true",
                    help="also capture two consecutive rounds into a HIP graph and time its replays; "
                         "value and ms_per_step then come from the replays (launch-bound small "
                         "workloads), the roofline still from the eager launches")
    ap.add_argument("--variant", default="",
                    help="comma-separated variant switches of the outer rule for the timed launches: "
                         "current_round, anchor_pull, norm_clip (fp32 transport only; not the headline)")
    ap.add_argument("--sweep-waves", type=int, default=0,
                    help="co2_params.sweep_waves_per_cu for the timed launches (0 = the library's default)")
    ap.add_argument("--side-waves", type=int, default=-1,
                    help="350m_overlap only: sweep_waves_per_cu of the side-stream outer update "
                         "(-1 = the schedule's default)")
    ap.add_argument("--inner-gemm-tflop", type=float, default=0.0,
                    help="350m_overlap only: run about this many TFLOP of bf16 GEMMs before each local step "
                         "as a compute-bound stand-in for the forward/backward pass (0 = none: the round is "
                         "then HBM-bound on both streams)")
    ap.add_argument("--own-in-place", action="store_true",
                    help="delta_out overwrites deltas[0] in place (one buffer for the worker's own "
                         "pseudo-gradient instead of a ping-pong pair)")
    ap.add_argument("--store-last-params", action="store_true",
                    help="350m_overlap only: the last local step of a round also stores x_{t,tau} "
                         "(4 more bytes per parameter; nothing reads it)")
    ap.add_argument("--plain-buffers", action="store_true",
                    help="350m_overlap only: separate plain allocations instead of one buffer set")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def _segment_chunks(table, limit):
    """Groups of whole consecutive segments of at most `limit` elements (a larger
    segment is a group of its own): (first element, last element + 1, re-based table)."""
    out, i, S = [], 0, len(table) - 1
    while i < S:
        j = i + 1
        while j < S and table[j + 1] - table[i] <= limit:
            j += 1
        out.append((table[i], table[j], [o - table[i] for o in table[i:j + 1]]))
        i = j
    return out


def cpu_baseline(cfg, table, bufs, t, min_seconds=10.0, max_passes=3):
    """The oracle, as it stands, on this host's cores, on the workload resident on the
    device: the round-t inputs (anchor, momentum, local params, the worker's own
    previous pseudo-gradient and the K-1 peers') are copied to host memory chunk by
    chunk (whole segments) and handed to the oracle; only the oracle calls are timed.
    Returns (single-thread figure over whole passes of the config, all-core figure)."""
    import os
    import threading

    import numpy as np
    import torch

    from oracle import co2_oracle

    a, m, x, own, peers = bufs
    cur = own[t % 2]
    dev_in = [x, a, m, cur] + list(peers)
    kw = dict(alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau, step=t)
    co2_oracle.build()
    co2_oracle.sqnorms(np.zeros(1, np.float32), [0, 1])          # load the library

    def staged(pinned, lo, hi):
        """Host copies (numpy views of pinned memory) of elements [lo, hi) of every input."""
        views = [pb[:hi - lo] for pb in pinned]
        for v, d in zip(views, dev_in):
            v.copy_(d[lo:hi], non_blocking=True)
        torch.cuda.synchronize()
        return [v.numpy() for v in views]

    def oracle_on(arrs, tab):
        co2_oracle.outer_step_f32(seg_off=tab, x=arrs[0], a=arrs[1], m=arrs[2], deltas=arrs[3:], **kw)

    # ---- single thread, whole passes over the configuration
    chunks = _segment_chunks(table, 1 << 26)
    big = max(hi - lo for lo, hi, _ in chunks)
    pinned = [torch.empty(big, dtype=torch.float32, pin_memory=True) for _ in dev_in]
    spent, done, passes = 0.0, 0, 0
    while passes < max_passes and spent < min_seconds:
        for lo, hi, tab in chunks:
            arrs = staged(pinned, lo, hi)
            t0 = time.perf_counter()
            oracle_on(arrs, tab)
            spent += time.perf_counter() - t0
            done += hi - lo
        passes += 1
    one = {"value": done / spent, "unit": "params/s", "cores": 1, "kind": "oracle", "sampled": False,
           "sample": f"{passes} whole pass(es) over all {len(table) - 1} segments ({table[-1]} params, K={cfg.K}) "
                     f"of the workload resident on the device, streamed in {len(chunks)} chunks of whole "
                     f"segments; {spent:.1f} s inside the oracle, g++ -O2, 1 thread"}
    del pinned

    # ---- all cores: one unchanged oracle call per thread, each on its own chunk
    cores = len(os.sched_getaffinity(0))
    small = [c for c in _segment_chunks(table, 1 << 24) if c[1] - c[0] <= 1 << 24]
    small.sort(key=lambda c: c[0] - c[1])
    picked = small[:cores]
    sets = []
    for lo, hi, tab in picked:
        pin = [torch.empty(hi - lo, dtype=torch.float32, pin_memory=True) for _ in dev_in]
        sets.append((staged(pin, lo, hi), tab, pin))
    best = None
    for _ in range(3):
        ths = [threading.Thread(target=oracle_on, args=(arrs, tab)) for arrs, tab, _ in sets]
        t0 = time.perf_counter()
        for th in ths:
            th.start()
        for th in ths:
            th.join()
        el = time.perf_counter() - t0
        best = el if best is None else min(best, el)
    total = sum(hi - lo for lo, hi, _ in picked)
    many = {"value": total / best, "unit": "params/s", "cores": len(picked), "nproc": cores,
            "kind": "oracle, one call per thread on disjoint chunks of whole segments (not a tuned baseline)",
            "sampled": True,
            "sample": f"{len(picked)} chunks ({total} of {table[-1]} params) run concurrently, best of 3"}
    return one, many


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
    use_set = not args.plain_buffers

    def make_grads(w):
        """tau bf16 gradient buffers: in the worker's buffer set when it has one."""
        bufs = ([v.view(torch.bfloat16) for v in w.extra] if use_set else
                [torch.empty(n, dtype=torch.bfloat16, device=dev) for _ in range(tau)])
        return [co2_inputs.fill_bf16_normal_(g, cfg.adamw["grad_std"], co2_inputs.seed_for(cfg.seed, 10 + k))
                for k, g in enumerate(bufs)]
    rounds = max(args.steps, 12)
    res = {}
    # Optional compute-bound stand-in for the forward/backward pass of each local step: a chain of
    # bf16 GEMMs (library calls, only a load generator here) of about --inner-gemm-tflop TFLOP.
    gemm = None
    if args.inner_gemm_tflop > 0:
        G = 8192
        ga, gb, gc = (torch.randn(G, G, dtype=torch.bfloat16, device=dev) * 0.01 for _ in range(3))
        reps = max(1, round(args.inner_gemm_tflop * 1e12 / (2 * G ** 3)))

        def gemm(_k):
            for _ in range(reps):
                torch.matmul(ga, gb, out=gc)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        gemm(0); torch.cuda.synchronize()
        e0.record(); gemm(0); e1.record(); torch.cuda.synchronize()
        gemm_ms = e0.elapsed_time(e1)
    for mode in ("serial", "overlapped"):
        w = CO2Worker(seg, K, tau, cfg.alpha, cfg.beta, cfg.phi, cfg.c, AdamWConfig(**hp), dev, init,
                      buffer_set=use_set, extra_bytes=[2 * n] * tau if use_set else ())
        grads = make_grads(w)
        if args.side_waves >= 0:
            w.side_waves = args.side_waves
        w.inner_compute = gemm
        w.skip_last_param_store = not args.store_last_params
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
        w_side_waves = w.side_waves
        del grads
        torch.cuda.synchronize()
        w.close()
        del w
        torch.cuda.empty_cache()
    # AdamW steps (the last one also reads the anchor and writes delta_out, and by default
    # does not store x_{t,tau}) + first-step norm slots (negligible) + split outer update
    bytes_round = (26 * tau + 8 - (0 if args.store_last_params else 4)) * n + (16 + 4 * K) * n
    out = {"metric": "overlapped round time (tau AdamW steps + outer update)",
           "value": res["overlapped"]["median_ms"], "unit": "ms", "n_gpus": 1, "steps": rounds,
           "warmup": 10, "ms_per_step": res["overlapped"]["median_ms"], "higher_is_better": False,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{cfg.name}: n={n}, K={K}, tau={tau}, bf16 grads, fp32 master",
                      "side_stream_sweep_waves_per_cu": w_side_waves,
                      "buffers": "one buffer set (64 MiB pieces)" if use_set else "separate plain allocations",
                      "last_local_step_stores_params": bool(args.store_last_params),
                      "algorithmic_bytes_per_param_per_round": bytes_round // n,
                      "compacted_gib": round(compacted / 2**30, 1)},
           "serial": res["serial"], "overlapped": res["overlapped"],
           "overlap_speedup": res["serial"]["median_ms"] / res["overlapped"]["median_ms"],
           "round_gbps_algorithmic": bytes_round / (res["overlapped"]["median_ms"] * 1e-3) / 1e9}
    if gemm is not None:
        out["config"]["inner_compute"] = {
            "kind": f"{reps} bf16 GEMM(s) {G}x{G}x{G} before each local step (stand-in for forward/backward)",
            "tflop_per_local_step": reps * 2 * G ** 3 / 1e12, "ms_per_local_step_alone": gemm_ms}
        del out["round_gbps_algorithmic"]          # the round is no longer HBM-bound
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
    bf16 = args.deltas != "f32"                     # 16-bit storage of the pseudo-gradients
    dd = dict(dtype={"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[args.deltas],
              device=dev)
    lam = torch.empty(S, **f32)
    ws = torch.empty(co2.workspace_bytes(n, S, K), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    carried = args.form == "carried"
    entry = {"f32": co2.co2_outer_step, "bf16": co2.co2_outer_step_bf16,
             "f16": co2.co2_outer_step_f16}[args.deltas]

    def typed(views):
        a, m, x = (v.view(torch.float32) for v in views[:3])
        ds = [v.view(dd["dtype"]) for v in views[3:]]
        return a, m, x, ds[:2], ds[2:]

    variant = [v for v in args.variant.split(",") if v]
    vflags = 0
    for v in variant:
        vflags |= {"current_round": co2.CO2_FLAG_CURRENT_ROUND, "anchor_pull": co2.CO2_FLAG_ANCHOR_PULL,
                   "norm_clip": co2.CO2_FLAG_NORM_CLIP}[v]
    # the current-round order keeps no previous own pseudo-gradient: Eq. 3's denominator comes
    # from first-inner-step norms (synthetic here: the drift scale)
    fsn = torch.full((S,), cfg.drift_scale, **f32) if "current_round" in variant else None

    def launch(bufs, t, ev=None, clipped=None, on=None):
        """One outer step of round t on stream `on` (default: the current stream)."""
        a, m, x, own, peers = bufs
        cur, nxt = own[t % 2], own[(t + 1) % 2]          # deltas[0] = last round's delta_out
        if args.own_in_place:
            cur = nxt = own[0]
        flags = (co2.CO2_FLAG_CARRIED_NORMS if (carried and t >= 2) else 0) | vflags
        p = co2.make_params(seg, K, cfg.alpha, cfg.beta, cfg.phi, cfg.c, cfg.tau, t, flags,
                            ev[0] if ev else None, ev[1] if ev else None,
                            None if "norm_clip" in variant else clipped,
                            pull_rho=0.5, sweep_waves_per_cu=args.sweep_waves)
        entry(p, x, a, a, m, [cur] + peers, nxt, fsn, lam, ws, stream=on or stream)

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
    layout = args.layout
    if layout == "separate":
        a = torch.empty(n, **f32); m = torch.empty(n, **f32); x = torch.empty(n, **f32)
        own = [torch.empty(n, **dd), torch.empty(n, **dd)]
        peers = [torch.empty(n, **dd) for _ in range(K - 1)]
    else:
        from paper_2401_16265_amd import placement as pl
        dbytes = n * (2 if bf16 else 4)
        sizes = [4 * n] * 3 + [dbytes] * (K + 1)
        pieces = tuple(int(v) << 20 for v in args.piece_mib.split(",")) if args.piece_mib else ()
        if layout == "piece-major":
            # The recommended layout, taken as it comes: no candidate is timed against another.
            # (The bench has the GPU to itself, so it may compact the free memory first.)
            try:
                placement = pl.choose_placement(sizes, probe, dev, candidates=0, probe_first=True,
                                                compact=True, pieces=(pieces or pl.DEFAULT_PIECES)[:1])
            except RuntimeError as exc:               # no virtual-memory support, or no room
                print(f"bench.py: piece-major buffer set unavailable ({exc}); falling back to "
                      "--layout search", file=sys.stderr)
                layout = "search"
        if layout == "search":
            placement = pl.choose_placement(sizes, probe, dev, candidates=max(1, args.placement_candidates),
                                            probe_first=True, compact=True, pieces=pieces,
                                            gaps=pl.DEFAULT_GAPS)
        elif layout == "first":
            placement = pl.choose_placement(sizes, None, dev, gaps=(pl.PAGE,))
        a, m, x, own, peers = typed(placement.views)
    student = cfg.drift == "student_t"

    def drift(t, bid, rnd=0):
        sd = co2_inputs.seed_for(cfg.seed, bid, rnd)
        dst = x if t.dtype != torch.float32 else t        # x doubles as fp32 scratch here
        if student:
            co2_inputs.fill_student_t_(dst, cfg.drift_scale, cfg.drift_nu, sd)
        else:
            co2_inputs.fill_normal_(dst, cfg.drift_scale, sd)
        if dst is not t:
            t.copy_(dst)

    def live_inputs(t):
        """What round t consumes besides the state the library carries: the K-1 peers'
        pseudo-gradients of round t-1 and this worker's local parameters after its inner
        loop (anchor + drift).  Drawn fresh for every round, outside every timed region."""
        for k, pb in enumerate(peers):
            drift(pb, 200 + k, t)
        drift(x, 100, t)
        x.add_(a)

    co2_inputs.fill_normal_(a, cfg.param_std, co2_inputs.seed_for(cfg.seed, 1))
    co2_inputs.fill_normal_(m, cfg.momentum_std, co2_inputs.seed_for(cfg.seed, 2))
    drift(own[0 if args.own_in_place else 1], 99)           # own pseudo-gradient of the round before round 1
    torch.cuda.synchronize()

    step_no = [1]
    bufs = (a, m, x, own, peers)
    warmup = max(args.warmup, 2 if carried else 0)   # carried sums exist from round 2 on
    for _ in range(warmup):
        live_inputs(step_no[0])
        launch(bufs, step_no[0])
        step_no[0] += 1
    torch.cuda.synchronize()

    # ---- timed rounds: per-round HIP events on the launch stream around the whole
    # step (all its kernels) and, inside the library, around the sweep kernel.
    step_ev = [(co2.HipEvent(), co2.HipEvent()) for _ in range(args.steps)]
    sweep_ev = [(co2.HipEvent(), co2.HipEvent()) for _ in range(args.steps)]
    clipped = torch.zeros(S, dtype=torch.int64, device=dev)
    lam_hist, graphs = [], {}
    if args.hip_graph:
        # one graph per half of the delta_out ping-pong; inputs are refreshed between replays
        side = torch.cuda.Stream()
        for par in (0, 1):
            graphs[par] = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graphs[par], stream=side):
                launch(bufs, 2 + par, on=torch.cuda.current_stream().cuda_stream)   # any round >= 2 of that parity
    wall0 = time.perf_counter()
    for i in range(args.steps):
        t = step_no[0]
        live_inputs(t)
        torch.cuda.synchronize()
        last = i == args.steps - 1
        step_ev[i][0].record(stream)
        if graphs:
            graphs[t % 2].replay()
        else:
            launch(bufs, t, sweep_ev[i], clipped if last else None)
        step_ev[i][1].record(stream)
        lam_hist.append(lam.clone())
        step_no[0] += 1
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0

    import statistics
    step_ms = [b.elapsed_ms(e) for b, e in step_ev]
    ms_per_step = statistics.median(step_ms)
    launch_mode = "hip graph replays (one graph per round parity)" if graphs else "eager"
    if graphs:
        # the sweep's own events cannot be recorded inside a captured launch: time a few eager rounds for the roofline
        sweep_ev = sweep_ev[:3]
        for i in range(3):
            live_inputs(step_no[0])
            launch(bufs, step_no[0], sweep_ev[i], clipped if i == 2 else None)
            step_no[0] += 1
        torch.cuda.synchronize()
        graphs.clear()
    # ---- cross-check: the same number of steps launched back to back inside one host-clock
    # bracket (synchronize on both sides).  Only the first of them consumes live inputs: without a
    # refresh in between, params == anchor afterwards and the later steps see zero drift, which is
    # why this figure is reported beside the per-round one and not as the metric.
    live_inputs(step_no[0])
    torch.cuda.synchronize()
    bb0 = time.perf_counter()
    for _ in range(args.steps):
        launch(bufs, step_no[0])
        step_no[0] += 1
    torch.cuda.synchronize()
    back_to_back_ms = (time.perf_counter() - bb0) * 1e3 / args.steps
    sweep_times = [b.elapsed_ms(e) for b, e in sweep_ev]
    sweep_ms = sum(sweep_times) / len(sweep_times)
    per_elem = (26 + 2 * K) if bf16 else (28 + 4 * K)   # algorithmic bytes per coordinate, one sweep
    if "current_round" in variant:
        per_elem -= 4                                    # deltas[0] is not read
    if "norm_clip" in variant:
        per_elem -= 8                                    # params and anchor are written by the second kernel
    sweep_bytes = per_elem * n
    achieved = sweep_bytes / (sweep_ms * 1e-3) / 1e9
    lam_all = torch.stack(lam_hist)
    lam_min, lam_max = float(lam_all.min()), float(lam_all.max())
    clipped_count = int(clipped.sum().item())

    # ---- yardstick: plain copy kernel over one buffer pair (8 B/element)
    cb, ce = co2.HipEvent(), co2.HipEvent()
    co2.co2_copy_f32(a, x, n, stream=stream)               # x is redrawn before its next use
    cb.record(stream)
    for _ in range(5):
        co2.co2_copy_f32(a, x, n, stream=stream)
    ce.record(stream)
    ce.synchronize()
    copy_gbps = 8 * n * 5 / (cb.elapsed_ms(ce) * 1e-3) / 1e9

    # a profiled constant exists only for Algorithm 1 in the carried form (what the profile ran)
    traffic_key = (cfg.name, args.deltas, K) if (not variant and carried) else None
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
                   "variant": variant or "none (Algorithm 1)",
                   "inputs": "local params and the K-1 peers' pseudo-gradients redrawn before every round, "
                             "untimed; the worker's own pseudo-gradient is the previous round's delta_out",
                   "timing": {"per": "round, HIP events on the launch stream around all kernels of the step",
                              "median_ms": ms_per_step, "min_ms": min(step_ms), "max_ms": max(step_ms),
                              "mean_ms": sum(step_ms) / len(step_ms),
                              "wall_s_including_input_generation": wall,
                              "back_to_back_ms_per_step_host_clock": back_to_back_ms},
                   "lambda_min": lam_min, "lambda_max": lam_max,
                   "clipped_coordinates_last_timed_step": clipped_count,
                   "layout": layout,
                   "placement": ("separate allocations" if placement is None else
                                 placement.report() if layout != "first" else "first allocation"),
                   "step_gbps_algorithmic": (per_elem + (0 if carried else (6 if bf16 else 8))) * n
                                            / (ms_per_step * 1e-3) / 1e9},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(traffic_key, (None, None))[0],
                     "traffic_source": MEASURED_TRAFFIC_BYTES.get(traffic_key, (None, None))[1],
                     "kernel": "fused_sweep", "kernel_ms": sweep_ms,
                     "kernel_ms_min": min(sweep_times), "kernel_ms_max": max(sweep_times),
                     "algorithmic_bytes": sweep_bytes, "copy_kernel_gbps": copy_gbps},
    }
    if not args.no_cpu_baseline and not bf16:
        t = step_no[0]
        live_inputs(t)
        torch.cuda.synchronize()
        out["cpu_baseline"], out["cpu_baseline_all_cores"] = cpu_baseline(cfg, table, bufs, t)
    del a, m, x, own, peers, bufs
    torch.cuda.synchronize()
    if placement is not None:
        placement.release()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
