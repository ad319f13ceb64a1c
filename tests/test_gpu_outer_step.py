"""GPU parity: the HIP library (through the C ABI) against the CPU oracle,
element by element, on the same seeded inputs.

Tolerance: every element of
every output within 1e-5 relative of the fp32-ordered oracle; Lambda and the
norms within 1e-5 relative; and, where the harness also carries the all-fp64
evaluation, within 1e-5 of it relative to the operands of each sum.  Both sides
evaluate the same unfused fp32 expression, so bit equality is the usual outcome
and is reported, but the assertion is the tolerance.
"""
import gc

import numpy as np
import pytest
import torch

import co2_inputs
import paper_2401_16265_amd as co2
from harness import HP, OuterStepHarness, assert_close
from streamed import StreamedOuterStepHarness

pytestmark = pytest.mark.gpu
INF = float("inf")


@pytest.fixture()
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    d = torch.device("cuda:0")
    yield d
    gc.collect()
    torch.cuda.empty_cache()


def run_steps(h, steps, **kw):
    out = []
    for _ in range(steps):
        print(f"  outer step t={h.t} n={h.n} S={h.S} K={h.hp.K} {kw}", flush=True)
        out.append(h.step(**kw))
    torch.cuda.synchronize()
    return out


# ------------------------------------------------------------------ config 1
def test_tiny_config(dev):
    cfg = co2_inputs.CONFIGS["tiny"]
    table = co2_inputs.config_table(cfg)
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau)
    h = OuterStepHarness(table, hp, dev, seed=cfg.seed, momentum_std=cfg.momentum_std,
                         truth=True, start_step=1)
    res = run_steps(h, 1)[0]
    assert res["lambda"] <= 1e-5 and np.all(h.last["lam"] > 1.0)
    print("tiny:", res)


def test_tiny_config_heavy_clipping(dev):
    cfg = co2_inputs.CONFIGS["tiny"]
    table = co2_inputs.config_table(cfg)
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=1e-3, c=cfg.c, tau=cfg.tau)
    h = OuterStepHarness(table, hp, dev, seed=3, momentum_std=0.02, truth=True, start_step=1)
    run_steps(h, 2)
    assert h.last["nclipped"] > h.n // 2
    # clipped coordinates moved by exactly alpha*phi
    moved = np.abs(h.gather(h.a).astype(np.float64) - h._truth_prev[0])
    assert moved.max() <= hp.alpha * hp.phi * (1 + 1e-4)


# ------------------------------------------------------------------ edge shapes
EDGE_TABLES = {
    "one_element": [0, 1],
    "five_two_segments": [0, 2, 5],
    "per_coordinate_1023": list(range(0, 1024)),
    "global_4097": [0, 4097],
    "odd_offsets_empty_segments": [0, 0, 13, 13, 2049, 5000, 5000, 6221],
    "boundary_at_tile_edges": [0, 2048, 4096, 4096, 8192, 8193, 16384 + 2048],
    "many_small_then_large": list(range(0, 300, 3)) + [300, 40000],
}


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
@pytest.mark.parametrize("K", [1, 2, 3, 8, 16])
def test_edge_shapes(dev, name, K):
    h = OuterStepHarness(EDGE_TABLES[name], HP(K=K, beta=0.8, phi=0.01, c=1.0, tau=3), dev,
                         seed=7, momentum_std=0.02, truth=True)
    run_steps(h, 3)


@pytest.mark.parametrize("K", [4, 5, 6, 7, 9, 10, 11, 12, 13, 14, 15])
def test_every_worker_count(dev, K):
    h = OuterStepHarness([0, 77, 5000, 20011], HP(K=K, beta=0.9, phi=0.5, c=1.0), dev, seed=K,
                         start_step=1)
    run_steps(h, 1)


@pytest.mark.parametrize("hp", [
    HP(K=4, c=0.0), HP(K=4, phi=INF), HP(K=4, beta=0.0), HP(K=4, alpha=0.25, c=3.0, tau=12),
    HP(K=1, c=0.0, phi=INF, beta=0.5, alpha=0.7),
], ids=["no_penalty", "no_clipping", "no_momentum", "alpha_c_tau", "momentum_sgd"])
def test_hyperparameter_corners(dev, hp):
    table = co2_inputs.gpt_table(layers=2, d=64, ffn=256, vocab=1001, ctx=32)
    h = OuterStepHarness(table, hp, dev, seed=11, momentum_std=0.01, truth=True)
    res = run_steps(h, 3)
    if hp.c == 0.0:
        assert np.all(h.lam.cpu().numpy() == 1.0)


def test_first_step_norm_supplied(dev):
    table = co2_inputs.gpt_table(layers=2, d=64, ffn=256, vocab=1001, ctx=32)
    h = OuterStepHarness(table, HP(K=8, phi=0.02, tau=6), dev, seed=12, truth=True,
                         use_first_step_norm=True)
    run_steps(h, 3)
    assert np.all(h.last["lam"] > 1.0)


# ------------------------------------------------------------------ multi-step, all forms
@pytest.mark.parametrize("mode", ["two_pass", "carried", "split", "split_carried_fsn"])
def test_multi_step_ragged_table(dev, mode):
    """Six consecutive rounds from t=0 on a ragged table whose offsets are not
    multiples of 4 (odd vocabulary), state carried on both sides."""
    table = co2_inputs.gpt_table(layers=3, d=97, ffn=385, vocab=3001, ctx=63)
    assert any(o % 4 for o in table)
    h = OuterStepHarness(table, HP(K=8, beta=0.95, phi=2e-3, c=1.0), dev, seed=21,
                         momentum_std=0.0, drift="student_t", truth=True,
                         use_first_step_norm=(mode == "split_carried_fsn"))
    for t in range(6):
        flags = co2.CO2_FLAG_CARRIED_NORMS if (mode in ("carried", "split_carried_fsn") and t >= 1) else 0
        print(f"  {mode} t={t}", flush=True)
        h.step(flags=flags, split=mode.startswith("split"))
    assert h.last["nclipped"] > 0


# ------------------------------------------------------------------ bf16 transport of the deltas
@pytest.mark.parametrize("mode", ["two_pass", "carried", "split"])
def test_bf16_deltas_multi_step(dev, mode):
    table = co2_inputs.gpt_table(layers=3, d=97, ffn=385, vocab=3001, ctx=63)
    h = OuterStepHarness(table, HP(K=8, beta=0.95, phi=2e-3, c=1.0), dev, seed=31,
                         momentum_std=0.0, drift="student_t", truth=True, bf16=True)
    for t in range(6):
        flags = co2.CO2_FLAG_CARRIED_NORMS if (mode == "carried" and t >= 1) else 0
        print(f"  bf16 {mode} t={t}", flush=True)
        h.step(flags=flags, split=(mode == "split"))
    assert h.last["nclipped"] > 0 and np.any(h.last["lam"] > 1.0)


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
@pytest.mark.parametrize("K", [1, 3, 16])
def test_bf16_deltas_edge_shapes(dev, name, K):
    h = OuterStepHarness(EDGE_TABLES[name], HP(K=K, beta=0.8, phi=0.01, c=1.0, tau=3), dev,
                         seed=8, momentum_std=0.02, truth=True, bf16=True)
    run_steps(h, 3)


def test_bf16_deltas_1p3b_every_element(dev):
    """Headline-size buffers with bf16 pseudo-gradient transport (42 B/param): every
    element of every output and every Lambda against the oracle, three consecutive
    rounds, the last one in the carried (single-pass) form; buffers in one buffer set as
    in the bench."""
    cfg = co2_inputs.CONFIGS["1p3b"]
    table = co2_inputs.config_table(cfg)
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau)
    h = StreamedOuterStepHarness(table, hp, dev, seed=cfg.seed, drift="student_t",
                                 drift_scale=cfg.drift_scale, drift_nu=cfg.drift_nu,
                                 momentum_std=cfg.momentum_std, start_step=1, bf16=True, buffer_set=True)
    assert h.ch.n == 1_343_868_928
    for i in range(3):
        res = h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if i >= 2 else 0)
        print(f"  1p3b bf16 step {h.t - 1}: {res}", flush=True)
    assert res["lam_max"] > 1.0
    h.close()


def test_carried_norms_equal_two_pass(dev):
    """The sums left by the sweep give the same Lambda as re-reading m and d0."""
    table = co2_inputs.gpt_table(layers=2, d=128, ffn=512, vocab=2001, ctx=32)
    hs = [OuterStepHarness(table, HP(K=4, phi=0.01), dev, seed=5, momentum_std=0.0)
          for _ in range(2)]
    for t in range(4):
        hs[0].step(flags=0)
        hs[1].step(flags=co2.CO2_FLAG_CARRIED_NORMS if t >= 1 else 0)
        if t >= 1:
            assert_close(hs[1].lam.cpu().numpy(), hs[0].lam.cpu().numpy(), "Lambda", tol=1e-6)
        assert torch.equal(hs[0].m, hs[1].m) and torch.equal(hs[0].a, hs[1].a)


@pytest.mark.parametrize("transport", ["f32", "bf16", "f16"])
def test_own_pseudo_gradient_updated_in_place(dev, transport):
    """delta_out == deltas[0]: one buffer for the worker's own pseudo-gradient.  Every output
    keeps the bits of the run with a ping-pong pair (which the other tests compare with the
    oracle), over four rounds, the last two in the carried form; tiles with segment boundaries
    and a ragged end included."""
    table = [0, 5, 5, 1300, 70000, 100003]
    n, S, K = table[-1], len(table) - 1, 3
    seg = co2.SegmentTable(table, dev)
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[transport]
    entry = {"f32": co2.co2_outer_step, "bf16": co2.co2_outer_step_bf16, "f16": co2.co2_outer_step_f16}[transport]
    f32 = dict(dtype=torch.float32, device=dev)

    def run(in_place):
        a = co2_inputs.fill_normal_(torch.empty(n, **f32), 0.02, co2_inputs.seed_for(9, 1))
        m = co2_inputs.fill_normal_(torch.empty(n, **f32), 0.02, co2_inputs.seed_for(9, 2))
        x = torch.empty(n, **f32)
        own = [torch.zeros(n, dtype=tdt, device=dev) for _ in range(1 if in_place else 2)]
        lam = torch.ones(S, **f32)                 # round 0 writes no Lambda
        ws = torch.empty(co2.workspace_bytes(n, S, K), dtype=torch.uint8, device=dev)
        outs = []
        for t in range(4):
            co2_inputs.fill_student_t_(x, 1e-3, 3, co2_inputs.seed_for(9, 100, t))
            x.add_(a)
            peers = [co2_inputs.fill_normal_(torch.empty(n, **f32), 1e-3, co2_inputs.seed_for(9, 200 + k, t)).to(tdt)
                     for k in range(K - 1)]
            cur, nxt = (own[0], own[0]) if in_place else (own[t % 2], own[(t + 1) % 2])
            p = co2.make_params(seg, K, 1.0, 0.9, 2e-3, 1.0, 4, t, co2.CO2_FLAG_CARRIED_NORMS if t >= 2 else 0)
            entry(p, x, a, a, m, [cur] + peers, nxt, None, lam, ws)
            torch.cuda.synchronize()
            outs.append([v.clone() for v in (x, a, m, nxt.view(torch.int16) if tdt != torch.float32 else nxt, lam)])
        return outs

    for t, (got, want) in enumerate(zip(run(True), run(False))):
        for name, g, w in zip(("params", "anchor", "momentum", "delta_out", "Lambda"), got, want):
            assert torch.equal(g, w), f"round {t}: {name} differs when delta_out overwrites deltas[0]"
    # partial overlap is still refused
    a = torch.zeros(n + 64, **f32)
    p = co2.make_params(seg, 1, 1.0, 0.9, 1.0, 1.0, 4, 1, 0)
    ws = torch.empty(co2.workspace_bytes(n, S, 1), dtype=torch.uint8, device=dev)
    buf = torch.zeros(n + 64, **f32)
    rc = co2.co2_outer_step(p, torch.zeros(n, **f32), a[:n], a[:n], torch.zeros(n, **f32), [buf[:n]], buf[4:n + 4],
                            None, torch.empty(S, **f32), ws, check=False)
    assert rc == co2.CO2_EINVAL


def test_resume_from_saved_state(dev):
    """Checkpoint/resume: the state that defines a round is anchor, momentum, the
    in-flight pseudo-gradients and the round index.  Restoring it into fresh
    buffers (fresh workspace, so one two-pass round before carried sums exist
    again) continues bit for bit like the uninterrupted run."""
    table = co2_inputs.gpt_table(layers=2, d=97, ffn=385, vocab=2001, ctx=31)
    mk = lambda: OuterStepHarness(table, HP(K=4, phi=2e-3, beta=0.95), dev, seed=9, momentum_std=0.0)  # noqa: E731
    ref, run = mk(), mk()
    for t in range(6):
        ref.step(flags=co2.CO2_FLAG_CARRIED_NORMS if t >= 1 else 0)
    for t in range(3):
        run.step(flags=co2.CO2_FLAG_CARRIED_NORMS if t >= 1 else 0)
    saved = dict(a=run.a.clone(), m=run.m.clone(), x=run.x.clone(),
                 own=[o.clone() for o in run.own], t=run.t)
    # "restart": overwrite every live buffer, then restore from the checkpoint
    for b in [run.a, run.m, run.x, run.ws] + run.own + run.peers:
        b.fill_(0) if b.dtype != torch.uint8 else b.fill_(255)
    run.a.copy_(saved["a"]); run.m.copy_(saved["m"]); run.x.copy_(saved["x"])
    for o, so in zip(run.own, saved["own"]):
        o.copy_(so)
    for t in range(3, 6):
        run.step(flags=co2.CO2_FLAG_CARRIED_NORMS if t >= 4 else 0)
    for name in ("a", "m", "x", "lam"):
        assert torch.equal(getattr(ref, name), getattr(run, name)), name


def test_outer_step_in_a_hip_graph(dev):
    """The call only enqueues kernels, so a caller may capture it in a HIP graph
    (no memset nodes are recorded).  Replays are compared with eager calls."""
    table = co2_inputs.gpt_table(layers=2, d=64, ffn=256, vocab=1001, ctx=32)
    seg = co2.SegmentTable(table, dev)
    n, S, K = seg.n, seg.S, 4
    g = torch.Generator(device=dev); g.manual_seed(3)
    rnd = lambda std: torch.randn(n, device=dev, generator=g) * std  # noqa: E731
    a0, m0 = rnd(0.02), rnd(0.01)
    deltas = [rnd(1e-3) for _ in range(K)]
    noise = [rnd(1e-3) for _ in range(4)]

    def fresh():
        return dict(a=a0.clone(), m=m0.clone(), x=a0.clone(), dout=torch.empty(n, device=dev),
                    lam=torch.empty(S, device=dev),
                    ws=torch.empty(co2.workspace_bytes(n, S, K), dtype=torch.uint8, device=dev))

    def call(st, step):
        p = co2.make_params(seg, K, 1.0, 0.9, 2e-3, 1.0, 4, step)
        co2.co2_outer_step(p, st["x"], st["a"], st["a"], st["m"], deltas, st["dout"], None,
                           st["lam"], st["ws"])

    eager, graphed = fresh(), fresh()
    side = torch.cuda.Stream(device=dev)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(graphed, 1)                                   # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    graphed = fresh()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(graphed, 1)
    graphed["a"].copy_(a0); graphed["m"].copy_(m0)          # capture does not execute
    for r in range(4):
        eager["x"].copy_(eager["a"] + noise[r]); graphed["x"].copy_(graphed["a"] + noise[r])
        call(eager, 1)
        graph.replay()
        torch.cuda.synchronize()
        for name in ("a", "m", "x", "dout", "lam"):
            assert torch.equal(eager[name], graphed[name]), f"replay {r}: {name}"


# ------------------------------------------------------------------ norms entry point
def test_pseudo_grad_norms(dev, oracle):
    table = [0, 0, 13, 2049, 8192, 8193, 70001]
    seg = co2.SegmentTable(table, dev)
    n, S = seg.n, seg.S
    g = torch.Generator(device=dev); g.manual_seed(5)
    bufs = [torch.randn(n, device=dev, generator=g) * (0.1 * (i + 1)) for i in range(5)]
    mom = torch.randn(n, device=dev, generator=g)
    ws = torch.empty(co2.workspace_bytes(n, S, 1), dtype=torch.uint8, device=dev)
    p = co2.make_params(seg, 1, 1.0, 0.9, 0.5, 1.0, 1, 0)
    for nb, use_m in [(5, True), (3, False), (0, True), (1, False), (2, True)]:
        rows = nb + (1 if use_m else 0)
        out = torch.full((rows, S), -1.0, dtype=torch.float64, device=dev)
        co2.co2_pseudo_grad_norms(p, bufs[:nb], mom if use_m else None, out, ws)
        got = out.cpu().numpy()
        for i in range(nb):
            assert_close(got[i], oracle.sqnorms(bufs[i].cpu().numpy(), table), f"buffer {i}", tol=1e-12)
        if use_m:
            assert_close(got[nb], oracle.sqnorms(mom.cpu().numpy(), table, phi=0.5), "momentum", tol=1e-12)
    # determinism: same bits on a second call
    out2 = torch.empty_like(out)
    co2.co2_pseudo_grad_norms(p, bufs[:2], mom, out2, ws)
    assert torch.equal(out, out2)


# ------------------------------------------------------------------ config 2, full size
def test_gpt2_small_ten_steps(dev):
    """All 124 439 808 elements and all 148 Lambda, ten consecutive rounds."""
    cfg = co2_inputs.CONFIGS["gpt2s"]
    table = co2_inputs.config_table(cfg)
    assert table[-1] == 124_439_808 and len(table) - 1 == 148
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau)
    h = StreamedOuterStepHarness(table, hp, dev, seed=cfg.seed, drift_scale=cfg.drift_scale,
                                 momentum_std=cfg.momentum_std, start_step=1, chunk_elems=1 << 24)
    assert cfg.steps == 10 and h.ch.n == table[-1]
    for i in range(cfg.steps):
        res = h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if i >= 1 else 0)
        print(f"  gpt2s step {h.t - 1}: {res}", flush=True)


# ------------------------------------------------------------------ config 3, headline size
def test_1p3b_headline_every_element_twenty_steps(dev):
    """The headline workload as stated: 1 343 868 928 parameters in 292 segments,
    K=8, Student-t drift, 20 consecutive outer rounds in the launch configuration
    the bench times (carried norms after the first two rounds; the flat buffers in one
    buffer set with 64 MiB pieces, in the bench's order).  EVERY element of
    params, anchor, momentum and delta_out and every Lambda and clipped count of
    every round is compared with the oracle, which carries its own full state."""
    cfg = co2_inputs.CONFIGS["1p3b"]
    table = co2_inputs.config_table(cfg)
    assert table[-1] == 1_343_868_928 and len(table) - 1 == 292 and cfg.steps == 20
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau)
    h = StreamedOuterStepHarness(table, hp, dev, seed=cfg.seed, drift="student_t",
                                 drift_scale=cfg.drift_scale, drift_nu=cfg.drift_nu,
                                 momentum_std=cfg.momentum_std, start_step=1, buffer_set=True)
    assert h.ch.n == table[-1] and len(h.ch.sample) == 292
    clipped_steps, lam_max = 0, 1.0
    for i in range(cfg.steps):
        res = h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if i >= 2 else 0)
        print(f"  1p3b step {h.t - 1}: {res}", flush=True)
        clipped_steps += res["nclipped"] > 0
        lam_max = max(lam_max, res["lam_max"])
    assert clipped_steps > 0, "the heavy-tailed drift should trigger the clamp on some rounds"
    assert lam_max > 1.0
    # Norms of ALL 292 segments at full size through the norms entry point, against the
    # oracle's ascending fp64 sums over the oracle's own momentum and pseudo-gradient.
    from oracle import co2_oracle
    own = h.own[h.t % 2]
    out = torch.empty(2, h.S, dtype=torch.float64, device=dev)
    p = co2.make_params(h.seg, hp.K, hp.alpha, hp.beta, hp.phi, hp.c, hp.tau, h.t)
    co2.co2_pseudo_grad_norms(p, [own], h.m, out, h.ws)
    got = out.cpu().numpy()
    print("  full-size norms of all segments vs oracle", flush=True)
    # The oracle adds up to 1.3e8 non-negative terms one after the other, so its own sum
    # is only good to about N * 2^-53 ~ 1e-8 relative (the device's tree order is tighter);
    # 1e-9 is four orders inside the 1e-5 bar.
    assert_close(got[0], co2_oracle.sqnorms(h.o_own, table), "sum of d0^2, all segments", tol=1e-9)
    assert_close(got[1], co2_oracle.sqnorms(h.o_m, table, phi=hp.phi),
                 "sum of Clip(m)^2, all segments", tol=1e-9)
    del own
    h.close()


# ------------------------------------------------------------------ more than 2^31 elements
def test_flat_index_beyond_2_to_31(dev):
    """64-bit indexing: a flat vector of 2^31 + 4099 elements (8.6 GB per buffer);
    the sampled segments sit at the start, across the 2^31 boundary and at the
    ragged end."""
    n = (1 << 31) + 4099
    table = [0, 1000, (1 << 31) - 5, (1 << 31) + 1000, n]
    h = OuterStepHarness(table, HP(K=2, beta=0.9, phi=2e-3, c=1.0), dev, seed=17, sample=[0, 2, 3],
                         momentum_std=0.01)
    for t in range(3):
        print(f"  n={n} step {h.t}", flush=True)
        h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if t >= 2 else 0)
    lam = h.lam.cpu().numpy()
    assert np.all(lam >= 1.0) and np.all(np.isfinite(lam))


# ------------------------------------------------------------------ config 4, ZeRO-style shard
@pytest.mark.parametrize("rank", [1, 0])
def test_7b_shard_partial_segments(dev, rank):
    """One 1/16 slice of the 7B table (first and last segments are partial tensors):
    all 421 150 976 elements, 20 consecutive rounds."""
    cfg = co2_inputs.CONFIGS["7b_shard"]
    table = co2_inputs.config_table(cfg, rank=rank)
    assert table[-1] == 421_150_976 and cfg.steps == 20
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau)
    h = StreamedOuterStepHarness(table, hp, dev, seed=cfg.seed + rank, drift_scale=cfg.drift_scale,
                                 momentum_std=cfg.momentum_std, start_step=1, chunk_elems=1 << 25)
    assert h.ch.n == table[-1]
    for i in range(cfg.steps):
        res = h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if i >= 1 else 0)
        print(f"  7b shard rank {rank} step {h.t - 1}: {res}", flush=True)
    assert res["lam_max"] > 1.0
