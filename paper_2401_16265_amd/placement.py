"""Choosing where the flat buffers of the outer update live in device memory.

The fused sweep streams 3 + K + 1 flat buffers in lock step.  On MI355X its
duration depends on how those streams fall onto HBM channels and banks relative
to each other, which is decided by the physical pages behind the buffers.
Measured at 1.3B parameters, K = 8: the same kernel on the same data runs
between 11.8 and 13.4 ms depending on the allocation it was given (a
single-stream copy runs equally fast in all of them; the byte gap between
consecutive buffers moves it by another +-1.5 %), and what the driver hands out
for a plain allocation depends on the allocation history of the machine.  It is
stable for the life of an allocation, and a training job allocates once.

Two kinds of layout are made here:

  * piece-major buffer sets (co2_buffer_set_create): every buffer's physical
    memory is obtained in pieces, piece j of all buffers before piece j+1, so
    that what the sweep touches at one time lies close together.  With 64 MiB
    pieces they have been at the fast end in every set made, on every machine
    state tried; this is the layout to use, taken as it comes (candidates=0:
    nothing is compared by timing);
  * plain single allocations with the buffers carved out back to back, made in
    turn while earlier ones are still held, so that each lands on other physical
    pages, each tried with a few gaps between consecutive buffers.  The caller's
    probe -- a few launches of the real kernel -- is timed on every candidate and
    the fastest is kept; everything else is freed.  Kept for comparison with the
    buffer sets: one such allocation in three is slow, and on a machine whose
    memory has seen many allocate/free cycles all of them are.

compact_device_memory (opt-in: it briefly takes nearly all free memory of the
device, so only for a process that has the GPU to itself) first brings the
driver's free memory back to one block.

This module holds host logic only (allocation, slicing, timing decisions); the
probe it is given runs the library's kernels.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import torch

PAGE = 4096
DEFAULT_GAPS = (PAGE, 11 * PAGE, 259 * PAGE)    # odd page counts; 0, 2 pages and 1 MiB measure 1-3 % slower
# Piece size of the piece-major buffer sets.  Measured at 1.3B parameters (fp32 buffers of 5.4 GB): sets with
# 64 MiB pieces were fast every time (three sets held together, several processes, K = 8, 12, 16), as were
# 48-70 MiB; 16 MiB and 128 MiB were consistently 4-5 % slower, 256 MiB - 2 GiB anything in between.
DEFAULT_PIECES = (64 << 20,)


def padded(nbytes: int) -> int:
    """Buffer size rounded up to whole 4 KiB pages."""
    return (nbytes + PAGE - 1) // PAGE * PAGE


def carve(arena: torch.Tensor, sizes: Sequence[int], gap: int) -> List[torch.Tensor]:
    """uint8 views of `arena`, one per entry of `sizes` (bytes), consecutive buffers
    `gap` bytes beyond the previous one's padded end."""
    views, off = [], 0
    for b in sizes:
        views.append(arena[off:off + b])
        off += padded(b) + gap
    if off - gap > arena.numel():
        raise ValueError("arena too small for the requested buffers")
    return views


def arena_bytes(sizes: Sequence[int], gap: int) -> int:
    return sum(padded(b) + gap for b in sizes)


def compact_device_memory(device, headroom: int = 3 << 30) -> int:
    """Allocates nearly all free device memory in ONE allocation and frees it again.

    The driver keeps freed memory as a patchwork of blocks that it merges lazily;
    after other processes (or this one) have allocated and freed many buffers, a
    new multi-gigabyte allocation is assembled from scattered blocks and the sweep
    runs 5-10 % slower on it.  A request that only fits if everything is merged
    makes the driver do that merge, and what is freed afterwards is one block
    again.  Measured: plain allocations that probed at 12.5-13.4 ms before this
    call probed at 11.9-12.0 ms (the first and third of three) right after it.
    Only for a device this process has to itself: for a moment nearly all free memory
    is taken, and another process allocating at that instant would fail.
    Returns the number of bytes that were taken (0 if nothing could be)."""
    if torch.device(device).type != "cuda":
        return 0
    torch.cuda.synchronize(device)
    torch.cuda.empty_cache()
    free = torch.cuda.mem_get_info(device)[0]
    for h in (headroom, 2 * headroom, 4 * headroom, 8 * headroom):
        if free <= h:
            break
        try:
            big = torch.empty(free - h, dtype=torch.uint8, device=device)
        except RuntimeError:                      # torch.cuda.OutOfMemoryError is a RuntimeError
            continue
        taken = big.numel()
        del big
        torch.cuda.empty_cache()
        return taken
    return 0


@dataclass
class Placement:
    owner: object                        # what holds the memory: a uint8 tensor or a BufferSet
    views: List[torch.Tensor]            # uint8 views, one per requested buffer
    kind: str = "arena"                  # "arena" or "piece-major"
    gap: int = PAGE                      # arena: bytes between consecutive buffers
    piece_bytes: int = 0                 # piece-major: requested piece size
    compacted_bytes: int = 0             # what compact_device_memory took before the search
    first_ms: Optional[float] = None     # probe of a plain allocation made BEFORE compaction and search
    pieces_ms: dict = field(default_factory=dict)                 # piece size -> probe ms (or error text)
    arenas_ms: List[List[float]] = field(default_factory=list)    # [candidate][gap index]
    gaps: Tuple[int, ...] = ()

    def report(self) -> dict:
        chosen = (f"piece-major, {self.piece_bytes >> 20} MiB pieces" if self.kind == "piece-major"
                  else f"arena, gap {self.gap} B")
        flat = [t for row in self.arenas_ms for t in row] + [v for v in self.pieces_ms.values()
                                                              if isinstance(v, float)]
        return {"first_allocation_ms": None if self.first_ms is None else round(self.first_ms, 3),
                "worst_candidate_ms": round(max(flat), 3) if flat else None,
                "compacted_gib": round(self.compacted_bytes / 2**30, 1),
                "piece_major_ms": {f"{k >> 20} MiB": (round(v, 3) if isinstance(v, float) else v)
                                   for k, v in self.pieces_ms.items()},
                "arenas_ms": [[round(t, 3) for t in row] for row in self.arenas_ms],
                "gaps_bytes": list(self.gaps), "chosen": chosen}

    def release(self):
        """Frees the memory; every use of the views has completed and been dropped."""
        self.views = []
        if hasattr(self.owner, "close"):
            self.owner.close()
        self.owner = None


def choose_placement(sizes: Sequence[int], probe: Optional[Callable[[List[torch.Tensor]], float]],
                     device, candidates: int = 4, gaps: Sequence[int] = DEFAULT_GAPS,
                     pieces: Sequence[int] = (), reserve_bytes: int = 4 << 30,
                     spacer_bytes: int = 192 << 20, buffer_set=None, compact: bool = False,
                     probe_first: bool = False) -> Placement:
    """Allocate buffers of `sizes` bytes where `probe` runs fastest.

    With `probe` None this is one plain allocation with the first gap.  Otherwise:
    compact_device_memory() first if `compact` is set (opt-in: it takes nearly all free
    device memory for a moment, which is only safe on a device this process has to
    itself), then
    up to `candidates` plain allocations, then one piece-major buffer set per
    entry of `pieces` (`buffer_set(sizes, piece, device)` -> object with .views
    and .close(); default: the library's BufferSet), each zero-filled and timed
    with `probe(views)` -> milliseconds (plain allocations once per gap).  While
    the next plain allocation is made, the best candidate so far and the latest
    loser stay allocated and a small spacer of growing size is added, so that
    every candidate is backed by different physical pages; at most three
    candidates are alive at once, fewer if device memory, less `reserve_bytes`,
    does not hold them.  The kept buffers contain whatever the probe left in them:
    initialise them afterwards.  `probe_first`: before anything else, also time the
    probe on one plain allocation exactly as the device hands it out (no compaction,
    first gap) and free it again -- the figure a caller gets who does none of this
    (reported as `first_ms`).
    """
    gaps = tuple(gaps)
    if not gaps:
        raise ValueError("need at least one gap")
    total = arena_bytes(sizes, max(gaps))
    if probe is None:
        arena = torch.empty(total, dtype=torch.uint8, device=device)
        return Placement(arena, carve(arena, sizes, gaps[0]), "arena", gaps[0], gaps=gaps)

    on_gpu = torch.device(device).type == "cuda"

    def room() -> bool:
        return not on_gpu or torch.cuda.mem_get_info(device)[0] >= total + reserve_bytes

    def drop(owner):
        if owner is not None and hasattr(owner, "close"):
            owner.close()

    first_ms = None
    if probe_first:
        arena = torch.empty(total, dtype=torch.uint8, device=device)
        arena.zero_()
        first_ms = float(probe(carve(arena, sizes, gaps[0])))
        del arena
        if on_gpu:
            torch.cuda.empty_cache()
    compacted = compact_device_memory(device) if compact else 0
    best = None          # (ms, Placement)
    loser = None         # the latest plain allocation that lost, kept until the next one exists
    pieces_ms, arenas_ms = {}, []

    def offer(ms: float, cand: Placement):
        """Keeps the faster of `best` and `cand`; returns the owner that lost."""
        nonlocal best
        if best is None or ms < best[0]:
            lost = best[1].owner if best else None
            best = (ms, cand)
            return lost
        return cand.owner

    spacers = []
    for ci in range(max(0, candidates)):
        if best is not None and not room():
            loser = None
            torch.cuda.empty_cache()
            if not room():
                break
        if ci and spacer_bytes:
            spacers.append(torch.empty(ci * spacer_bytes, dtype=torch.uint8, device=device))
        arena = torch.empty(total, dtype=torch.uint8, device=device)
        arena.zero_()
        row = [float(probe(carve(arena, sizes, g))) for g in gaps]
        arenas_ms.append(row)
        gi = min(range(len(gaps)), key=row.__getitem__)
        # the loser before this one goes back to the driver below
        loser = offer(row[gi], Placement(arena, carve(arena, sizes, gaps[gi]), "arena", gaps[gi]))
        del arena
        torch.cuda.empty_cache()
    loser = None
    torch.cuda.empty_cache()

    if buffer_set is None and on_gpu and pieces:
        from .binding import BufferSet as buffer_set
    for piece in (pieces if buffer_set is not None else ()):
        if best is not None and not room():
            break
        try:
            bs = buffer_set(sizes, piece, device)
        except RuntimeError as exc:                     # no such memory left, or no support
            pieces_ms[piece] = f"failed: {exc}"
            continue
        for v in bs.views:
            v.zero_()
        ms = float(probe(list(bs.views)))
        pieces_ms[piece] = ms
        drop(offer(ms, Placement(bs, list(bs.views), "piece-major", piece_bytes=piece)))

    if best is None:
        raise RuntimeError("no candidate placement could be allocated")
    kept = best[1]
    del best, loser, spacers
    torch.cuda.empty_cache()
    kept.pieces_ms, kept.arenas_ms, kept.gaps = pieces_ms, arenas_ms, gaps
    kept.compacted_bytes = compacted
    kept.first_ms = first_ms
    return kept
