"""co2_buffer_set on the GPU: the buffers are ordinary flat device memory (every
byte readable and writable, no two buffers overlap, piece boundaries are
invisible), the outer update gives bit-identical results on them and on plain
allocations, and the memory comes back on destroy."""
import gc

import numpy as np
import pytest
import torch

import co2_inputs
import paper_2401_16265_amd as co2

pytestmark = pytest.mark.gpu
MIB = 1 << 20


def test_buffers_are_flat_disjoint_and_reusable():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    dev = torch.device("cuda:0")
    n = 1_600_003                                         # 6.4 MB fp32: several 2 MiB pieces, odd tail
    sizes = [4 * n, 4 * n, 2 * n, 4 * n, 1]
    free_after = []
    for round_ in range(3):
        print(f"  buffer set round {round_}", flush=True)
        bs = co2.BufferSet(sizes, 2 * MIB, dev)
        assert len(bs.views) == len(sizes)
        spans = sorted((p, p + b) for p, b in zip(bs.ptrs, sizes))
        for (lo0, hi0), (lo1, _hi1) in zip(spans, spans[1:]):
            assert hi0 <= lo1, "buffers overlap"
        assert all(p % 4096 == 0 for p in bs.ptrs)
        for i, v in enumerate(bs.views):
            assert v.dtype == torch.uint8 and v.numel() == sizes[i] and v.data_ptr() == bs.ptrs[i]
        # distinct patterns through every byte, including the piece boundaries
        for i, v in enumerate(bs.views):
            idx = torch.arange(v.numel(), device=dev, dtype=torch.int64)
            v.copy_(((idx * (2 * i + 3) + i) % 251).to(torch.uint8))
        torch.cuda.synchronize()
        for i, v in enumerate(bs.views):
            idx = np.arange(v.numel(), dtype=np.int64)
            assert np.array_equal(v.cpu().numpy(), ((idx * (2 * i + 3) + i) % 251).astype(np.uint8)), i
        del v, idx
        bs.close()
        bs.close()                                        # idempotent
        gc.collect()
        torch.cuda.empty_cache()
        free_after.append(torch.cuda.mem_get_info(dev)[0])
    # the first round also loads torch's kernels; a set is 24 MB: later rounds must not lose that much
    assert free_after[2] >= free_after[1] - 8 * MIB, f"memory did not come back: {free_after}"


def test_outer_step_is_bit_identical_on_a_buffer_set():
    dev = torch.device("cuda:0")
    table = [0, 5, 300_000, 300_000, 1_000_001, 1_600_003]
    seg = co2.SegmentTable(table, dev)
    n, S, K = seg.n, seg.S, 3
    f32 = dict(dtype=torch.float32, device=dev)
    names = ["x", "a", "m", "own0", "own1"] + [f"peer{k}" for k in range(K - 1)]
    plain = {nm: torch.empty(n, **f32) for nm in names}
    bs = co2.BufferSet([4 * n] * len(names), 2 * MIB, dev)
    placed = {nm: v.view(torch.float32) for nm, v in zip(names, bs.views)}
    for j, nm in enumerate(names):
        co2_inputs.fill_normal_(plain[nm], 0.02 if nm in ("x", "a") else 1e-3, co2_inputs.seed_for(9, j))
        placed[nm].copy_(plain[nm])
    outs = []
    for bufs in (plain, placed):
        lam = torch.empty(S, **f32)
        ws = torch.empty(co2.workspace_bytes(n, S, K), dtype=torch.uint8, device=dev)
        for t in (1, 2, 3):
            flags = co2.CO2_FLAG_CARRIED_NORMS if t >= 2 else 0
            p = co2.make_params(seg, K, 1.0, 0.9, 1.5e-3, 1.0, 4, t, flags)
            cur, nxt = bufs[f"own{t % 2}"], bufs[f"own{(t + 1) % 2}"]
            co2.co2_outer_step(p, bufs["x"], bufs["a"], bufs["a"], bufs["m"],
                               [cur] + [bufs[f"peer{k}"] for k in range(K - 1)], nxt, None, lam, ws)
        torch.cuda.synchronize()
        outs.append({nm: bufs[nm].clone() for nm in ("x", "a", "m", "own0", "own1")} | {"lam": lam})
    for nm in outs[0]:
        assert torch.equal(outs[0][nm], outs[1][nm]), f"{nm} differs between plain and placed buffers"
    del placed, bufs, cur, nxt
    bs.close()
