"""The placement chooser on the GPU: compaction takes and returns device memory, and
choose_placement runs end to end with a real probe (launches of the outer update)
over plain allocations and piece-major buffer sets, keeping buffers that work."""
import gc

import pytest
import torch

import co2_inputs
import paper_2401_16265_amd as co2
from paper_2401_16265_amd import placement as pl

pytestmark = pytest.mark.gpu
MIB = 1 << 20


def test_compaction_takes_and_returns_memory():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    dev = torch.device("cuda:0")
    torch.zeros(1, device=dev)                      # context and kernels loaded before measuring
    gc.collect()
    torch.cuda.empty_cache()
    free0 = torch.cuda.mem_get_info(dev)[0]
    print(f"  compacting {free0 >> 30} GiB free", flush=True)
    taken = pl.compact_device_memory(dev)
    free1 = torch.cuda.mem_get_info(dev)[0]
    assert taken >= free0 // 2, (taken, free0)
    assert free1 >= free0 - 64 * MIB, (free0, free1)


@pytest.mark.parametrize("pieces", [(), (2 * MIB,)])
def test_choose_placement_with_a_real_probe(pieces):
    dev = torch.device("cuda:0")
    table = [0, 300_000, 1_000_001, 1_200_000]
    seg = co2.SegmentTable(table, dev)
    n, S, K = seg.n, seg.S, 2
    lam = torch.empty(S, dtype=torch.float32, device=dev)
    ws = torch.empty(co2.workspace_bytes(n, S, K), dtype=torch.uint8, device=dev)
    calls = []

    def step(views, t):
        x, a, m, own0, own1, peer = (v.view(torch.float32) for v in views)
        own = (own0, own1)
        p = co2.make_params(seg, K, 1.0, 0.9, 1.0, 1.0, 4, t, 0)
        co2.co2_outer_step(p, x, a, a, m, [own[t % 2], peer], own[(t + 1) % 2], None, lam, ws)

    def probe(views):
        b, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        step(views, 1)
        b.record()
        step(views, 2)
        e.record()
        e.synchronize()
        calls.append(views[0].data_ptr())
        return b.elapsed_time(e)

    sizes = [4 * n] * 6
    placed = pl.choose_placement(sizes, probe, dev, candidates=2, gaps=(pl.PAGE, 2 * pl.PAGE),
                                 pieces=pieces, compact=False)
    rep = placed.report()
    print("  placement report:", rep, flush=True)
    assert len(rep["arenas_ms"]) == 2 and all(len(r) == 2 for r in rep["arenas_ms"])
    assert len(rep["piece_major_ms"]) == len(pieces)
    assert all(isinstance(v, float) for v in rep["piece_major_ms"].values())
    assert len(calls) == 4 + len(pieces)
    assert placed.kind in ("arena", "piece-major") and len(placed.views) == 6
    # the kept buffers are usable: one more round on real values
    for j, v in enumerate(placed.views):
        co2_inputs.fill_normal_(v.view(torch.float32), 1e-3, co2_inputs.seed_for(3, j))
    step(placed.views, 3)
    torch.cuda.synchronize()
    assert torch.isfinite(placed.views[0].view(torch.float32)).all()
    placed.release()
    gc.collect()
    torch.cuda.empty_cache()
