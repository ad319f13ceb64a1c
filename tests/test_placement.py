"""Host logic of the buffer-placement chooser (no GPU: CPU tensors, a scripted probe)."""
import pytest
import torch

from paper_2401_16265_amd import placement as pl


def test_carve_offsets_and_alignment():
    sizes = [4 * 1000, 4 * 1000, 2 * 1000, 4097]
    gap = 8192
    arena = torch.zeros(pl.arena_bytes(sizes, gap), dtype=torch.uint8)
    views = pl.carve(arena, sizes, gap)
    assert [v.numel() for v in views] == sizes
    base = arena.data_ptr()
    offs = [v.data_ptr() - base for v in views]
    assert offs[0] == 0
    for i in range(1, len(sizes)):
        assert offs[i] - offs[i - 1] == pl.padded(sizes[i - 1]) + gap
        assert offs[i] % pl.PAGE == 0
    # views do not overlap and reinterpret cleanly
    views[0].view(torch.float32).fill_(1.0)
    views[1].view(torch.float32).fill_(2.0)
    assert float(views[0].view(torch.float32).sum()) == 1000.0
    assert int(views[2].sum()) == 0


def test_carve_rejects_small_arena():
    with pytest.raises(ValueError):
        pl.carve(torch.zeros(10000, dtype=torch.uint8), [8192, 8192], 4096)


def test_plain_allocation_without_probe():
    p = pl.choose_placement([4096, 100], None, "cpu", candidates=3, gaps=(4096,))
    assert p.chosen == (0, 0) and p.probe_ms == [] and len(p.views) == 2
    assert p.report()["candidates_ms"] == []


def test_fastest_candidate_and_gap_is_kept():
    script = iter([5.0, 4.0, 6.0,    # candidate 0, three gaps
                   3.5, 2.5, 9.0,    # candidate 1
                   7.0, 7.0, 7.0])   # candidate 2
    seen = []

    def probe(views):
        seen.append((views[0].data_ptr(), views[1].data_ptr() - views[0].data_ptr()))
        assert int(views[0].sum()) == 0          # candidates arrive zero-filled
        return next(script)

    sizes = [8192, 8192, 100]
    p = pl.choose_placement(sizes, probe, "cpu", candidates=3, gaps=(4096, 8192, 12288))
    assert p.chosen == (1, 1) and p.gap == 8192
    assert len(seen) == 9
    assert p.views[0].data_ptr() == seen[4][0]                   # candidate 1's memory
    assert p.views[1].data_ptr() - p.views[0].data_ptr() == 8192 + 8192
    assert p.report() == {"candidates_ms": [[5.0, 4.0, 6.0], [3.5, 2.5, 9.0], [7.0, 7.0, 7.0]],
                          "gaps_bytes": [4096, 8192, 12288], "chosen": [1, 1]}
    # the three candidates were distinct allocations held at the same time
    assert len({s[0] for s in seen}) == 3
