"""Host logic of the whole-vector parity harness: the chunking of a segment table
into groups of whole segments must cover every sampled element exactly once and
keep each chunk's re-based table consistent (no GPU, no oracle)."""
import numpy as np
import pytest

import co2_inputs
from streamed import SegmentChunks


@pytest.mark.parametrize("table,sample,chunk", [
    ([0, 1], None, 4),
    ([0, 0, 13, 13, 2049, 5000, 5000, 6221], None, 1000),
    ([0, 0, 13, 13, 2049, 5000, 5000, 6221], [1, 4, 6], 10),
    (co2_inputs.gpt_table(layers=2, d=64, ffn=256, vocab=1001, ctx=32), None, 20000),
    (co2_inputs.gpt_table(layers=2, d=64, ffn=256, vocab=1001, ctx=32), [0, 3, 4, 5, 20, 27], 5000),
    (co2_inputs.config_table(co2_inputs.CONFIGS["1p3b"]), None, 1 << 26),
])
def test_chunks_partition_the_sample(table, sample, chunk):
    ch = SegmentChunks(table, sample, chunk)
    segs = list(range(len(table) - 1)) if sample is None else sorted(set(sample))
    assert ch.sample == segs
    assert ch.n == sum(table[s + 1] - table[s] for s in segs)
    # chunks tile the compact segment and element ranges in order
    assert ch.chunks[0].i0 == 0 and ch.chunks[-1].i1 == len(segs)
    assert ch.chunks[0].c0 == 0 and ch.chunks[-1].c1 == ch.n
    covered = []
    for a, b in zip(ch.chunks, ch.chunks[1:]):
        assert a.i1 == b.i0 and a.c1 == b.c0
    for c in ch.chunks:
        assert c.table[0] == 0 and c.table[-1] == c.elems and np.all(np.diff(c.table) >= 0)
        assert len(c.table) == c.i1 - c.i0 + 1
        assert sum(hi - lo for lo, hi in c.runs) == c.elems
        # a chunk exceeds the limit only if it is a single oversized segment (plus empty ones)
        if c.elems > chunk:
            assert np.count_nonzero(np.diff(c.table)) == 1
        # the runs are exactly the device ranges of the chunk's segments, in order
        want = [(table[segs[i]], table[segs[i] + 1]) for i in range(c.i0, c.i1)
                if table[segs[i] + 1] > table[segs[i]]]
        flat = [j for lo, hi in want for j in (lo, hi)]
        merged = [j for lo, hi in c.runs for j in (lo, hi)]
        # merging adjacent ranges removes pairs of equal inner endpoints only
        assert merged[0] == flat[0] and merged[-1] == flat[-1] if flat else not merged
        covered += c.runs
    assert sorted(ch.order) == list(range(len(ch.chunks)))
    sizes = [ch.chunks[q].elems for q in ch.order]
    assert sizes == sorted(sizes, reverse=True)
    assert ch.max_chunk == max(sizes)
    # no device element is staged twice
    covered.sort()
    for (l0, h0), (l1, h1) in zip(covered, covered[1:]):
        assert h0 <= l1
