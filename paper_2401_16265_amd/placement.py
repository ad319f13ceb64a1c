"""Choosing where the flat buffers of the outer update live in device memory.

The fused sweep streams 3 + K + 1 flat buffers in lock step.  On MI355X its
duration depends on how those streams fall onto HBM channels and banks relative
to each other, which is decided by (a) the physical pages behind the allocation
and (b) the byte distance between consecutive buffers.  Measured at 1.3B
parameters, K = 8: the same kernel on the same data runs between 11.9 and 13.4 ms
depending on the allocation it was given (a single-stream copy runs equally fast
in all of them), and the gap between buffers moves it by another +-3 %.  Neither
can be predicted from user space, but both are stable for the life of an
allocation, and a training job allocates once.  So the layout is chosen by
measurement: a few candidate allocations are held at the same time (so that they
are backed by different physical pages), the caller's probe -- a few launches of
the real kernel -- is timed on each candidate with each gap, and the fastest is
kept; the others are freed.

This module holds host logic only (allocation, slicing, timing decisions); the
probe it is given runs the library's kernels.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import torch

PAGE = 4096
DEFAULT_GAPS = (PAGE, 2 * PAGE, (1 << 20) + PAGE)


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


@dataclass
class Placement:
    arena: torch.Tensor                  # the allocation that was kept (uint8)
    gap: int                             # chosen gap between consecutive buffers, bytes
    views: List[torch.Tensor]            # uint8 views, one per requested buffer
    probe_ms: List[List[float]] = field(default_factory=list)   # [candidate][gap index]
    gaps: Tuple[int, ...] = ()
    chosen: Tuple[int, int] = (0, 0)     # (candidate, gap index)

    def report(self) -> dict:
        return {"candidates_ms": [[round(t, 3) for t in row] for row in self.probe_ms],
                "gaps_bytes": list(self.gaps), "chosen": list(self.chosen)}


def choose_placement(sizes: Sequence[int], probe: Optional[Callable[[List[torch.Tensor]], float]],
                     device, candidates: int = 3, gaps: Sequence[int] = DEFAULT_GAPS,
                     reserve_bytes: int = 4 << 30) -> Placement:
    """Allocate the buffers of `sizes` bytes out of one device allocation.

    With `probe` None or candidates <= 1 and one gap, this is a plain single
    allocation.  Otherwise up to `candidates` allocations are made and held
    together (fewer if device memory, less `reserve_bytes`, does not hold them),
    each is zero-filled, `probe(views)` -> milliseconds is called for every
    (allocation, gap) pair, and the fastest pair is kept.  The kept buffers
    contain whatever the probe left in them: initialise them afterwards.
    """
    gaps = tuple(gaps)
    if not gaps:
        raise ValueError("need at least one gap")
    total = arena_bytes(sizes, max(gaps))
    if probe is None or (candidates <= 1 and len(gaps) == 1):
        arena = torch.empty(total, dtype=torch.uint8, device=device)
        return Placement(arena, gaps[0], carve(arena, sizes, gaps[0]), [], gaps, (0, 0))

    arenas: List[torch.Tensor] = []
    times: List[List[float]] = []
    for _ in range(max(1, candidates)):
        if arenas and torch.device(device).type == "cuda":
            free, _total = torch.cuda.mem_get_info(device)
            if free < total + reserve_bytes:
                break
        arena = torch.empty(total, dtype=torch.uint8, device=device)
        arena.zero_()
        arenas.append(arena)
        times.append([float(probe(carve(arena, sizes, g))) for g in gaps])
    best = min(((t, ci, gi) for ci, row in enumerate(times) for gi, t in enumerate(row)))
    _, ci, gi = best
    kept = arenas[ci]
    del arenas, arena
    torch.cuda.empty_cache()              # hand the other candidates back to the driver
    return Placement(kept, gaps[gi], carve(kept, sizes, gaps[gi]), times, gaps, (ci, gi))
