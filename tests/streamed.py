"""Whole-vector parity at the workloads' real sizes: the HIP library against the
CPU oracle on EVERY element, streamed in chunks of whole segments.

The device holds the full workload.  The oracle side holds its own full state
(anchor, momentum, own pseudo-gradient) in host memory and advances it chunk by
chunk: segments are independent in the update, so a group of whole segments with
a re-based segment table is itself a valid, smaller problem for the oracle, and
several such groups can be handed to the (single-threaded, unchanged) oracle
from several host threads at once.  Per chunk a worker thread

  1. copies the chunk of every INPUT both sides consume (the local drift, the
     peers' pseudo-gradients -- all drawn by co2_inputs on the device) to host
     memory (through small pinned bounce buffers),
  2. runs the oracle on it, in place on the oracle's own state,
  3. copies the chunk of every OUTPUT the device produced and compares it with
     the oracle's, element by element (bit equality first; where bits differ,
     the 1e-5 relative bar).

Data only ever flows device -> host as inputs or for comparison; nothing the HIP
library computed is fed to the oracle.
"""
from __future__ import annotations

import queue
import threading
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

import co2_inputs
import paper_2401_16265_amd as co2
from harness import HP, REL_TOL, rel_err
from oracle import co2_oracle


@dataclass
class Chunk:
    i0: int                          # compact segment range [i0, i1)
    i1: int
    c0: int                          # compact element range [c0, c1)
    c1: int
    runs: List[Tuple[int, int]]      # device element ranges, in order, that make up [c0, c1)
    table: np.ndarray                # segment table of the chunk, re-based to 0

    @property
    def elems(self) -> int:
        return self.c1 - self.c0


class SegmentChunks:
    """A sample of whole segments (default: all of them) of a device-sized table,
    packed into a compact index space and cut into chunks of consecutive sampled
    segments of at most `chunk_elems` elements (a larger segment is a chunk of its
    own)."""

    def __init__(self, table: Sequence[int], sample: Optional[Sequence[int]], chunk_elems: int):
        self.table = [int(o) for o in table]
        S = len(self.table) - 1
        self.sample = list(range(S)) if sample is None else sorted(set(sample))
        sizes = [self.table[s + 1] - self.table[s] for s in self.sample]
        self.otable = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        self.n = int(self.otable[-1])
        self.chunks: List[Chunk] = []
        i = 0
        while i < len(self.sample):
            j, total = i, 0
            while j < len(self.sample) and (j == i or total + sizes[j] <= chunk_elems):
                total += sizes[j]
                j += 1
            runs: List[Tuple[int, int]] = []
            for k in range(i, j):
                lo, hi = self.table[self.sample[k]], self.table[self.sample[k] + 1]
                if hi == lo:
                    continue
                if runs and runs[-1][1] == lo:
                    runs[-1] = (runs[-1][0], hi)
                else:
                    runs.append((lo, hi))
            c0, c1 = int(self.otable[i]), int(self.otable[j])
            self.chunks.append(Chunk(i, j, c0, c1, runs, (self.otable[i:j + 1] - c0).astype(np.int64)))
            i = j
        self.max_chunk = max(c.elems for c in self.chunks)
        # largest first: the thread pool then balances better
        self.order = sorted(range(len(self.chunks)), key=lambda q: -self.chunks[q].elems)


# Staging memory.  The chunk-sized host arrays the oracle works on are ordinary
# (pageable) numpy arrays, kept in one pool for the whole process and grown on
# demand; device data reaches them through two small pinned bounce buffers per
# worker thread (64 MiB each), so the amount of pinned memory stays at about a
# gigabyte whatever the chunk size.
_POOL = {"sets": [], "nbuf": 0, "nbytes": 0}
_POOL_LOCK = threading.Lock()
BOUNCE_BYTES = 64 << 20


def staging_sets(nsets: int, nbuf: int, nbytes: int) -> "queue.Queue":
    """A queue of `nsets` sets of `nbuf` uint8 host arrays of at least `nbytes` bytes."""
    with _POOL_LOCK:
        if _POOL["nbuf"] < nbuf or _POOL["nbytes"] < nbytes or len(_POOL["sets"]) < nsets:
            nb = max(nbuf, _POOL["nbuf"])
            by = max(nbytes, _POOL["nbytes"])
            ns = max(nsets, len(_POOL["sets"]))
            _POOL["sets"] = []                 # drop the old blocks before taking larger ones
            _POOL["sets"] = [[np.zeros(by, dtype=np.uint8) for _ in range(nb)] for _ in range(ns)]
            _POOL["nbuf"], _POOL["nbytes"] = nb, by
        q: "queue.Queue" = queue.Queue()
        for s in _POOL["sets"][:nsets]:
            q.put(s)
        return q


_TLS = threading.local()
_BOUNCE_LOCK = threading.Lock()
_BOUNCE_FREE: list = []          # pinned buffer pairs of threads that have ended


class _Lane:
    """Per-thread copy stream and pinned bounce buffers (returned to a free list when
    the thread object dies, so a new thread pool does not pin new memory)."""

    def __init__(self):
        with _BOUNCE_LOCK:
            self.bounce = _BOUNCE_FREE.pop() if _BOUNCE_FREE else None
        if self.bounce is None:
            self.bounce = [torch.empty(BOUNCE_BYTES, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
        self.stream = torch.cuda.Stream()      # default priority
        self.done = [torch.cuda.Event(), torch.cuda.Event()]

    def __del__(self):
        with _BOUNCE_LOCK:
            _BOUNCE_FREE.append(self.bounce)


def _lane() -> _Lane:
    if not hasattr(_TLS, "lane"):
        _TLS.lane = _Lane()
    return _TLS.lane


def stage(dev_buf: torch.Tensor, chunk: Chunk, dest: np.ndarray, ready: torch.cuda.Event) -> np.ndarray:
    """Chunk of a device buffer -> typed view of the host array `dest` (16-bit float
    buffers come back as their uint16 bit patterns).  Waits for `ready` on the device
    first.  The data travels in pieces through the thread's pinned bounce buffers: the
    copy of one piece from the device overlaps the host copy of the previous one."""
    if dev_buf.dtype in (torch.bfloat16, torch.float16):
        dev_buf = dev_buf.view(torch.int16)
    width = dev_buf.element_size()
    np_dtype = {4: np.float32, 2: np.uint16}[width]
    out = dest[:chunk.elems * width].view(np_dtype)
    lane = _lane()
    per = BOUNCE_BYTES // width
    pieces = []
    off = 0
    for lo, hi in chunk.runs:
        for p0 in range(lo, hi, per):
            p1 = min(p0 + per, hi)
            pieces.append((p0, p1, off))
            off += p1 - p0
    pending = None
    with torch.cuda.stream(lane.stream):
        lane.stream.wait_event(ready)
        for i, (p0, p1, o) in enumerate(pieces):
            b = lane.bounce[i % 2].view(dev_buf.dtype)[:p1 - p0]
            b.copy_(dev_buf[p0:p1], non_blocking=True)
            lane.done[i % 2].record(lane.stream)
            if pending is not None:
                pb, po, pe = pending
                pe.synchronize()
                out[po:po + pb.numel()] = pb.numpy().view(np_dtype)
            pending = (b, o, lane.done[i % 2])
    if pending is not None:
        pb, po, pe = pending
        pe.synchronize()
        out[po:po + pb.numel()] = pb.numpy().view(np_dtype)
    return out


def for_each_chunk(chunks: SegmentChunks, fn, workers: int):
    """fn(chunk) for every chunk on a pool of host threads; the first exception wins."""
    with ThreadPoolExecutor(max_workers=workers) as ex:
        futs = [ex.submit(fn, chunks.chunks[q]) for q in chunks.order]
        for f in futs:
            f.result()


def same_or_close(got: np.ndarray, want: np.ndarray, what: str, stats: dict):
    """Bit equality, else the 1e-5 relative bar element by element."""
    if np.array_equal(got, want):
        return
    stats["bit_exact"] = False
    e = rel_err(got, want)
    stats["worst"] = max(stats.get("worst", 0.0), e)
    assert e <= REL_TOL, f"{what}: max relative error {e:.3e} > {REL_TOL:g}"


class StreamedOuterStepHarness:
    """co2_outer_step / co2_outer_step_bf16 over consecutive rounds, compared with
    the oracle on every element of the sampled segments (default: all segments)."""

    def __init__(self, table: Sequence[int], hp: HP, device, seed: int = 0,
                 sample: Optional[Sequence[int]] = None, drift: str = "normal",
                 drift_scale: float = 1e-3, drift_nu: int = 3, param_std: float = 0.02,
                 momentum_std: float = 0.02, start_step: int = 1, bf16: bool = False,
                 transport: Optional[str] = None, chunk_elems: int = 1 << 26, workers: int = 8,
                 nonstale: bool = False, norm_clip: bool = False, pull_rho: float = 1.0,
                 use_first_step_norm: bool = False, buffer_set: bool = False):
        """buffer_set: the flat device buffers come from one co2.BufferSet with the default piece
        size, in bench.py's order (anchor, momentum, params, own x 2, peers) -- the layout the
        bench times -- instead of separate plain allocations; close() frees it."""
        self.nonstale, self.norm_clip, self.pull_rho = nonstale, norm_clip, pull_rho
        self.variant = nonstale or norm_clip or pull_rho != 1.0
        self.table = [int(o) for o in table]
        self.n, self.S = self.table[-1], len(self.table) - 1
        self.transport = transport or ("bf16" if bf16 else "f32")
        bf16 = self.transport != "f32"                   # 16-bit storage of the pseudo-gradients
        self.hp, self.dev, self.seed, self.bf16 = hp, device, seed, bf16
        self.drift, self.drift_scale, self.drift_nu = drift, drift_scale, drift_nu
        self.workers = workers
        co2_oracle.build()                               # before any worker thread needs it
        co2_oracle.sqnorms(np.zeros(1, np.float32), [0, 1])
        self.seg = co2.SegmentTable(self.table, device)
        self.ch = SegmentChunks(self.table, sample, chunk_elems)
        n, K = self.n, hp.K
        f32 = dict(dtype=torch.float32, device=device)
        dd = dict(dtype={"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.transport],
                  device=device)
        self._set = None
        if buffer_set:
            esz = 2 if bf16 else 4
            self._set = co2.BufferSet([4 * n] * 3 + [esz * n] * (K + 1), 0, device)
            self.a, self.m, self.x = (v.view(torch.float32) for v in self._set.views[:3])
            flat = [v.view(dd["dtype"]).zero_() for v in self._set.views[3:]]
            self.own, self.peers = flat[:2], flat[2:]
        else:
            self.x, self.a, self.m = (torch.empty(n, **f32) for _ in range(3))
            self.own = [torch.zeros(n, **dd), torch.zeros(n, **dd)]
            self.peers = [torch.zeros(n, **dd) for _ in range(K - 1)]
        self.noise = torch.empty(n, **f32)          # this round's local drift (an input of both sides)
        self.lam = torch.empty(self.S, **f32)
        self.clipped = torch.full((self.S,), -1, dtype=torch.int64, device=device)
        self.ws = torch.empty(co2.workspace_bytes(n, self.S, K), dtype=torch.uint8, device=device)
        co2_inputs.fill_normal_(self.a, param_std, co2_inputs.seed_for(seed, 1))
        if momentum_std > 0:
            co2_inputs.fill_normal_(self.m, momentum_std, co2_inputs.seed_for(seed, 2))
        else:
            self.m.zero_()
        self.t = self.t0 = start_step
        self.fsn = torch.empty(self.S, **f32) if use_first_step_norm else None
        assert not (self.variant and bf16)
        # staging: the K-1 peers + the drift as inputs; outputs reuse the same arrays afterwards
        self.sets = staging_sets(workers, max(K, 4), 4 * self.ch.max_chunk)
        # ---- oracle state over the compact index space
        nc = self.ch.n
        self.o_a = np.empty(nc, dtype=np.float32)
        self.o_m = np.empty(nc, dtype=np.float32)
        self.o_own = np.zeros(nc, dtype=np.uint16 if bf16 else np.float32)
        self.o_x = np.empty(nc, dtype=np.float32) if pull_rho != 1.0 else None   # pulled local parameters
        if start_step >= 1 and not nonstale:
            # no earlier round produced the worker's own previous pseudo-gradient: drawn like a peer's
            self._fill_drift(self.own[start_step % 2], 99)
        ready = torch.cuda.Event()
        ready.record()

        def init(c: Chunk):
            st = self.sets.get()
            try:
                self.o_a[c.c0:c.c1] = stage(self.a, c, st[0], ready)
                self.o_m[c.c0:c.c1] = stage(self.m, c, st[1], ready)
                if start_step >= 1 and not nonstale:
                    self.o_own[c.c0:c.c1] = stage(self.own[start_step % 2], c, st[2], ready)
            finally:
                self.sets.put(st)
        for_each_chunk(self.ch, init, workers)

    def close(self):
        """Frees the buffer set, if the buffers were taken from one (all work on them has finished)."""
        if self._set is not None:
            torch.cuda.synchronize()
            self.x = self.a = self.m = self.own = self.peers = None
            self._set.close()
            self._set = None

    def _fill_drift(self, t: torch.Tensor, buffer_id: int):
        sd = co2_inputs.seed_for(self.seed, buffer_id, self.t)
        dst = self.noise if t.dtype != torch.float32 else t
        if self.drift == "student_t":
            co2_inputs.fill_student_t_(dst, self.drift_scale, self.drift_nu, sd)
        else:
            co2_inputs.fill_normal_(dst, self.drift_scale, sd)
        if dst is not t:
            t.copy_(dst)                          # the sender's rounding to bf16 (input synthesis)

    def step(self, flags: int = 0) -> dict:
        """One outer round on both sides; every sampled element compared.  Returns
        dict(bit_exact, worst, nclipped, lam_min, lam_max)."""
        hp, t, K = self.hp, self.t, self.hp.K
        cur, nxt = self.own[t % 2], self.own[(t + 1) % 2]       # cur: deltas[0]; nxt: delta_out
        if t >= 1 or self.nonstale:
            for k, pbuf in enumerate(self.peers):               # before the drift: bf16 peers are drawn through `noise`
                self._fill_drift(pbuf, 200 + k)
        self._fill_drift(self.noise, 100)
        pulled = self.pull_rho != 1.0 and t > self.t0           # local parameters carried over, not restarted
        torch.add(self.x if pulled else self.a, self.noise, out=self.x)   # inner loop stand-in
        o_fsn = None
        if self.fsn is not None:
            co2_inputs.fill_normal_(self.fsn, 1.0, co2_inputs.seed_for(self.seed, 300, t))
            self.fsn.abs_().mul_(self.drift_scale * 10).add_(self.drift_scale)
            o_fsn = self.fsn[self.ch.sample].cpu().numpy().copy()
        if self.nonstale:
            flags |= co2.CO2_FLAG_CURRENT_ROUND
        if self.norm_clip:
            flags |= co2.CO2_FLAG_NORM_CLIP
        if self.pull_rho != 1.0:
            flags |= co2.CO2_FLAG_ANCHOR_PULL
        p = co2.make_params(self.seg, K, hp.alpha, hp.beta, hp.phi, hp.c, hp.tau, t, flags,
                            clipped_out=None if self.norm_clip else self.clipped, pull_rho=self.pull_rho)
        entry = {"f32": co2.co2_outer_step, "bf16": co2.co2_outer_step_bf16,
                 "f16": co2.co2_outer_step_f16}[self.transport]
        entry(p, self.x, self.a, self.a, self.m, [None if self.nonstale else cur] + self.peers, nxt,
              self.fsn, self.lam, self.ws)
        ready = torch.cuda.Event()
        ready.record()
        params_equal_anchor = torch.equal(self.x, self.a)       # both hold x_{t+1,0}

        S_c = len(self.ch.sample)
        o_lam = np.ones(S_c, dtype=np.float32)
        o_clip = np.zeros(S_c, dtype=np.int64)
        o_scale = np.ones(S_c, dtype=np.float32)
        stats = {"bit_exact": True, "worst": 0.0}
        lock = threading.Lock()
        oracle_step = {"f32": co2_oracle.outer_step_f32, "bf16": co2_oracle.outer_step_bf16,
                       "f16": co2_oracle.outer_step_f16}[self.transport]
        phi32 = np.float32(hp.phi)

        def work(c: Chunk):
            st = self.sets.get()
            try:
                sl = slice(c.c0, c.c1)
                start = self.o_x[sl] if pulled else self.o_a[sl]
                o_x = start + stage(self.noise, c, st[0], ready)             # same fp32 add as on the device
                o_d = None
                if t >= 1 or self.nonstale:
                    o_d = [self.o_own[sl]] + [stage(pb, c, st[1 + k], ready)
                                              for k, pb in enumerate(self.peers)]
                kw = dict(seg_off=c.table, alpha=hp.alpha, beta=hp.beta, phi=hp.phi, c=hp.c, tau=hp.tau,
                          step=t, x=o_x, a=self.o_a[sl], m=self.o_m[sl], deltas=o_d,
                          first_step_norm=None if o_fsn is None else o_fsn[c.i0:c.i1])
                if self.variant:
                    if self.nonstale:
                        o_d[0] = np.full(c.elems, 1e3, np.float32)           # poison: must not be read
                    out = co2_oracle.outer_step_variant_f32(nonstale=self.nonstale, norm_clip=self.norm_clip,
                                                            pull_rho=self.pull_rho, **kw)
                else:
                    out = oracle_step(**kw)
                self.o_own[sl] = out["dout"]
                local = {"bit_exact": True, "worst": 0.0}
                if self.o_x is not None:
                    self.o_x[sl] = o_x
                    same_or_close(stage(self.x, c, st[3], ready), o_x, "params", local)
                else:
                    assert np.array_equal(o_x, self.o_a[sl]), "oracle: params and anchor must both hold x_{t+1,0}"
                same_or_close(stage(self.a, c, st[0], ready), self.o_a[sl], "anchor", local)
                same_or_close(stage(self.m, c, st[1], ready), self.o_m[sl], "momentum", local)
                g_d = stage(nxt, c, st[2], ready)
                if self.bf16:
                    assert np.array_equal(g_d, out["dout"]), "delta_out (16-bit patterns) differs"
                else:
                    same_or_close(g_d, out["dout"], "delta_out", local)
                if self.variant:
                    o_scale[c.i0:c.i1] = out["scale"]
                o_lam[c.i0:c.i1] = out["lam"]
                if (t >= 1 or self.nonstale) and not self.norm_clip:
                    om = self.o_m[sl]
                    for i in range(c.i0, c.i1):
                        lo, hi = int(c.table[i - c.i0]), int(c.table[i - c.i0 + 1])
                        o_clip[i] = np.count_nonzero(np.abs(om[lo:hi]) > phi32)
                    assert int(o_clip[c.i0:c.i1].sum()) == out["nclipped"]
                with lock:
                    stats["bit_exact"] &= local["bit_exact"]
                    stats["worst"] = max(stats["worst"], local["worst"])
            finally:
                self.sets.put(st)

        for_each_chunk(self.ch, work, self.workers)
        torch.cuda.synchronize()
        if self.pull_rho == 1.0:
            assert params_equal_anchor, "device: params and anchor must both hold x_{t+1,0}"
        if not self.norm_clip:
            g_clip = self.clipped[self.ch.sample].cpu().numpy()
            assert np.array_equal(g_clip, o_clip), "clipped-coordinate counts differ"
        else:
            stats["rescaled_segments"] = int(np.count_nonzero(o_scale < 1.0))
        if t >= 1 or self.nonstale:
            g_lam = self.lam[self.ch.sample].cpu().numpy()
            e = rel_err(g_lam, o_lam)
            assert e <= REL_TOL, f"Lambda: max relative error {e:.3e}"
            stats["lambda_err"] = e
        stats.update(nclipped=int(o_clip.sum()), lam_min=float(o_lam.min()), lam_max=float(o_lam.max()),
                     elements=self.ch.n, segments=S_c)
        self.o_lam = o_lam
        self.t += 1
        return stats
