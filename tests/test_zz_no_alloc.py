"""co2_outer_step_static -- the entry point for callers that cannot allocate --
against co2_outer_step on the same inputs, through the C ABI.

The two entry points run the same kernels in the same order; the only
difference is where the partial sums live (the library's per-GPU scratch array
instead of a caller workspace), so every output must be bit-equal.  Two calls in
a row share the scratch array, the second on a smaller problem; a carried-norms
sequence then checks that what one call leaves in the array is what the next
round reads.
"""
import pytest
import torch

import co2_inputs
import paper_2401_16265_amd as co2

pytestmark = pytest.mark.gpu


class Problem:
    """Identical inputs for both entry points; `ref` state goes through
    co2_outer_step, `sta` state through co2_outer_step_static."""

    def __init__(self, table, K, dev, seed):
        self.seg = co2.SegmentTable(table, dev)
        self.K, self.dev, self.seed = K, dev, seed
        n, S = self.seg.n, self.seg.S
        f32 = dict(dtype=torch.float32, device=dev)
        a = co2_inputs.fill_normal_(torch.empty(n, **f32), 0.02, co2_inputs.seed_for(seed, 1))
        m = co2_inputs.fill_normal_(torch.empty(n, **f32), 0.01, co2_inputs.seed_for(seed, 2))
        self.peers = [co2_inputs.fill_normal_(torch.empty(n, **f32), 1e-3, co2_inputs.seed_for(seed, 200 + k))
                      for k in range(K - 1)]
        own = co2_inputs.fill_normal_(torch.empty(n, **f32), 1e-3, co2_inputs.seed_for(seed, 99))
        self.state = {}
        for name in ("ref", "sta"):
            self.state[name] = dict(a=a.clone(), m=m.clone(), x=torch.empty(n, **f32),
                                    own=[own.clone(), torch.zeros(n, **f32)],
                                    lam=torch.full((S,), -1.0, **f32),
                                    clipped=torch.full((S,), -1, dtype=torch.int64, device=dev))
        self.ws = torch.empty(co2.workspace_bytes(n, S, K), dtype=torch.uint8, device=dev)

    def round(self, t, flags=0):
        """Round t >= 1 on both states; asserts bit equality of every output."""
        noise = co2_inputs.fill_normal_(torch.empty(self.seg.n, dtype=torch.float32, device=self.dev),
                                        1e-3, co2_inputs.seed_for(self.seed, 100, t))
        for name, st in self.state.items():
            cur, nxt = st["own"][(t + 1) % 2], st["own"][t % 2]
            torch.add(st["a"], noise, out=st["x"])
            p = co2.make_params(self.seg, self.K, 1.0, 0.9, 2e-3, 1.0, 4, t, flags,
                                clipped_out=st["clipped"])
            args = (p, st["x"], st["a"], st["a"], st["m"], [cur] + self.peers, nxt, None, st["lam"])
            if name == "ref":
                co2.co2_outer_step(*args, self.ws)
            else:
                co2.co2_outer_step_static(*args)
        torch.cuda.synchronize()
        r, s = self.state["ref"], self.state["sta"]
        for key in ("a", "m", "x", "lam", "clipped"):
            assert torch.equal(r[key], s[key]), f"round {t}: {key} differs"
        assert torch.equal(r["own"][t % 2], s["own"][t % 2]), f"round {t}: delta_out differs"
        assert bool((s["lam"] >= 1.0).all()) and int(s["clipped"].sum()) > 0


def test_static_scratch_matches_workspace_entry_point():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    dev = torch.device("cuda:0")
    big = co2_inputs.gpt_table(layers=3, d=97, ffn=385, vocab=3001, ctx=63)       # ragged, odd offsets
    small = [0, 5, 300, 300, 4099]
    assert big[-1] > 100 * small[-1]
    print(f"  static scratch: n={big[-1]} then n={small[-1]}", flush=True)
    Problem(big, 8, dev, seed=41).round(1)
    Problem(small, 3, dev, seed=42).round(1)          # second call, smaller input, same scratch array
    # carried sums live in the scratch array between two calls on the same problem
    pb = Problem(big, 8, dev, seed=43)
    pb.round(1)
    pb.round(2, co2.CO2_FLAG_CARRIED_NORMS)
    pb.round(3, co2.CO2_FLAG_CARRIED_NORMS)


def test_static_scratch_rejects_sizes_beyond_its_limit():
    """Argument checks happen on the host before anything is enqueued."""
    dev = torch.device("cuda:0")
    n = 200_000_000                                   # needs more than CO2_STATIC_SCRATCH_BYTES
    assert co2.workspace_bytes(n, 1, 2) > co2.CO2_STATIC_SCRATCH_BYTES
    seg = co2.SegmentTable([0, n], dev)
    tiny = torch.zeros(64, device=dev)                # never touched: the call is rejected first
    p = co2.make_params(seg, 2, 1.0, 0.9, 1.0, 1.0, 4, 1)
    rc = co2.co2_outer_step_static(p, tiny, tiny.clone(), tiny.clone(), tiny.clone(),
                                   [tiny.clone(), tiny.clone()], tiny.clone(), None, None, check=False)
    assert rc == co2.CO2_ESCRATCH
    assert "scratch" in co2.strerror(rc)
