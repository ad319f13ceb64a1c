"""Host logic of the buffer-placement chooser (no GPU: CPU tensors, a scripted probe,
a stand-in for the piece-major buffer set)."""
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
    assert p.kind == "arena" and p.gap == 4096 and len(p.views) == 2
    assert p.report()["arenas_ms"] == [] and p.report()["piece_major_ms"] == {}
    p.release()
    assert p.owner is None and p.views == []


def test_fastest_arena_and_gap_is_kept():
    script = iter([5.0, 4.0, 6.0,    # candidate 0, three gaps
                   3.5, 2.5, 9.0,    # candidate 1
                   7.0, 7.0, 7.0])   # candidate 2
    seen = []

    def probe(views):
        seen.append((views[0].data_ptr(), views[1].data_ptr() - views[0].data_ptr()))
        assert int(views[0].sum()) == 0          # candidates arrive zero-filled
        return next(script)

    sizes = [8192, 8192, 100]
    p = pl.choose_placement(sizes, probe, "cpu", candidates=3, gaps=(4096, 8192, 12288), pieces=())
    assert p.kind == "arena" and p.gap == 8192
    assert len(seen) == 9
    assert p.views[0].data_ptr() == seen[4][0]                   # candidate 1's memory
    assert p.views[1].data_ptr() - p.views[0].data_ptr() == 8192 + 8192
    assert p.report() == {"first_allocation_ms": None, "worst_candidate_ms": 9.0,
                          "compacted_gib": 0.0, "piece_major_ms": {},
                          "arenas_ms": [[5.0, 4.0, 6.0], [3.5, 2.5, 9.0], [7.0, 7.0, 7.0]],
                          "gaps_bytes": [4096, 8192, 12288], "chosen": "arena, gap 8192 B"}
    # the three candidates were distinct allocations held at the same time
    assert len({s[0] for s in seen}) == 3


class FakeSet:
    """Stand-in for the library's BufferSet: separate host tensors, records close()."""
    made, closed = [], []

    def __init__(self, sizes, piece, device):
        self.piece = piece
        self.views = [torch.full((b,), 9, dtype=torch.uint8) for b in sizes]
        FakeSet.made.append(piece)

    def close(self):
        FakeSet.closed.append(self.piece)


def test_piece_major_candidates_compete_with_arenas():
    FakeSet.made, FakeSet.closed = [], []
    mib = 1 << 20
    times = iter([2.5, 2.6,            # two arenas, one gap each
                  3.0, 2.0])           # piece-major sets: 4 MiB, 2 MiB

    def probe(views):
        assert all(int(v.max()) == 0 for v in views)
        return next(times)

    p = pl.choose_placement([4096, 512], probe, "cpu", candidates=2, gaps=(4096,),
                            pieces=(4 * mib, 2 * mib), buffer_set=FakeSet)
    assert p.kind == "piece-major" and p.piece_bytes == 2 * mib
    assert FakeSet.made == [4 * mib, 2 * mib] and FakeSet.closed == [4 * mib]   # the loser was freed
    assert p.report()["piece_major_ms"] == {"4 MiB": 3.0, "2 MiB": 2.0}
    assert p.report()["arenas_ms"] == [[2.5], [2.6]]
    assert p.report()["chosen"] == "piece-major, 2 MiB pieces"
    p.release()
    assert FakeSet.closed == [4 * mib, 2 * mib]


def test_arena_beats_piece_major_and_failed_sets_are_reported():
    FakeSet.made, FakeSet.closed = [], []
    mib = 1 << 20

    def flaky(sizes, piece, device):
        if piece == 8 * mib:
            raise RuntimeError("out of memory")
        return FakeSet(sizes, piece, device)

    times = iter([1.0, 3.0])           # the arena, then the one set that could be made
    p = pl.choose_placement([4096], lambda v: next(times), "cpu", candidates=1, gaps=(4096,),
                            pieces=(8 * mib, 2 * mib), buffer_set=flaky)
    assert p.kind == "arena"
    assert FakeSet.closed == [2 * mib]
    rep = p.report()
    assert rep["piece_major_ms"]["8 MiB"].startswith("failed") and rep["piece_major_ms"]["2 MiB"] == 3.0


def test_compaction_is_a_no_op_off_the_gpu():
    assert pl.compact_device_memory("cpu") == 0


def test_first_allocation_is_probed_before_the_search():
    """probe_first: one plain allocation, first gap, timed before compaction and
    search, reported beside the candidates."""
    script = iter([8.5, 5.0, 4.0, 3.0, 6.0])
    calls = []

    def probe(views):
        calls.append(views[1].data_ptr() - views[0].data_ptr())
        return next(script)

    p = pl.choose_placement([4096, 4096], probe, "cpu", candidates=2, gaps=(4096, 8192), pieces=(),
                            probe_first=True)
    assert calls[0] == 4096 + 4096                       # the first gap
    assert len(calls) == 5
    rep = p.report()
    assert rep["first_allocation_ms"] == 8.5 and rep["worst_candidate_ms"] == 6.0
    assert p.gap == 4096 and rep["arenas_ms"] == [[5.0, 4.0], [3.0, 6.0]]


def test_diagnostic_modules_import_without_a_gpu():
    """The two diagnostics only sequence launches: importing them needs no GPU, and their source
    names nothing under oracle/."""
    import importlib
    import inspect
    for name in ("paper_2401_16265_amd.placement_contrast", "paper_2401_16265_amd.cache_ceiling_probe"):
        mod = importlib.import_module(name)
        assert callable(mod.main)
        assert "oracle" not in inspect.getsource(mod)
