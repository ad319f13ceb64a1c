"""GPU parity of the variant switches of the outer rule (current-round mean,
anchor pull, clipping by norm rescale) and of binary16 transport, against the
CPU oracle, element by element.  Same bar as the base path: 1e-5 relative per
element and per Lambda (bit equality is the usual outcome and is reported)."""
import gc

import numpy as np
import pytest
import torch

import co2_inputs
import paper_2401_16265_amd as co2
from harness import HP, OuterStepHarness
from streamed import StreamedOuterStepHarness
from test_gpu_outer_step import EDGE_TABLES

pytestmark = pytest.mark.gpu
INF = float("inf")

VARIANTS = {
    "current_round": dict(nonstale=True),
    "anchor_pull": dict(pull_rho=0.3),
    "norm_clip": dict(norm_clip=True),
    "current_round+norm_clip": dict(nonstale=True, norm_clip=True),
    "all_three": dict(nonstale=True, norm_clip=True, pull_rho=0.75),
    "pull+norm_clip": dict(norm_clip=True, pull_rho=0.5),
}


@pytest.fixture()
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    d = torch.device("cuda:0")
    yield d
    gc.collect()
    torch.cuda.empty_cache()


def steps(h, n, carried_from=None):
    res = None
    for i in range(n):
        flags = co2.CO2_FLAG_CARRIED_NORMS if (carried_from is not None and i >= carried_from and h.t >= 1) else 0
        print(f"  t={h.t} n={h.n} S={h.S} K={h.hp.K} flags={flags} nonstale={h.nonstale} "
              f"norm_clip={h.norm_clip} rho={h.pull_rho}", flush=True)
        res = h.step(flags=flags)
    torch.cuda.synchronize()
    return res


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
@pytest.mark.parametrize("variant", sorted(VARIANTS))
@pytest.mark.parametrize("K", [1, 3, 8])
def test_variant_edge_shapes(dev, name, variant, K):
    v = VARIANTS[variant]
    # a penalty in the current-round order needs the first-step norms
    h = OuterStepHarness(EDGE_TABLES[name], HP(K=K, beta=0.8, phi=0.01, c=1.0, tau=3), dev, seed=51,
                         momentum_std=0.02, use_first_step_norm=v.get("nonstale", False), **v)
    steps(h, 3)


@pytest.mark.parametrize("K", list(range(1, 17)))
def test_current_round_every_worker_count(dev, K):
    h = OuterStepHarness([0, 77, 5000, 20011], HP(K=K, beta=0.9, phi=0.5, c=0.0), dev, seed=60 + K,
                         nonstale=True)
    steps(h, 2)


@pytest.mark.parametrize("variant", sorted(VARIANTS))
@pytest.mark.parametrize("form", ["two_pass", "carried"])
def test_variant_multi_step_ragged_table(dev, variant, form):
    """Six consecutive rounds from t=0 on a ragged table with odd offsets, state
    carried on both sides, heavy-tailed drift so that clamp / rescale both bite."""
    v = VARIANTS[variant]
    table = co2_inputs.gpt_table(layers=3, d=97, ffn=385, vocab=3001, ctx=63)
    h = OuterStepHarness(table, HP(K=8, beta=0.95, phi=0.05 if v.get("norm_clip") else 2e-3, c=1.0), dev,
                         seed=52, momentum_std=0.0, drift="student_t",
                         use_first_step_norm=v.get("nonstale", False), **v)
    steps(h, 6, carried_from=1 if form == "carried" else None)
    assert np.any(h.last["lam"] > 1.0)
    if v.get("norm_clip"):
        sc = h.last["scale"]
        assert np.any(sc < 1.0) and np.any(sc == 1.0), "the rescale should bite on some segments only"
    else:
        assert h.last["nclipped"] > 0


def test_slow_momentum_form(dev):
    """Section 3.2's recursion as it stands before the staleness: current-round
    pseudo-gradients, no penalty, no clipping; carried form from the second round."""
    table = co2_inputs.gpt_table(layers=2, d=64, ffn=256, vocab=1001, ctx=32)
    h = OuterStepHarness(table, HP(K=4, alpha=0.7, beta=0.8, phi=INF, c=0.0), dev, seed=53,
                         momentum_std=0.0, nonstale=True)
    steps(h, 5, carried_from=1)
    assert np.all(h.lam.cpu().numpy() == 1.0) and h.last["nclipped"] == 0


def test_anchor_pull_with_rho_one_is_the_plain_restart(dev):
    table = [0, 300, 4099]
    hs = [OuterStepHarness(table, HP(K=3, phi=0.01), dev, seed=54, momentum_std=0.01) for _ in range(2)]
    for t in range(3):
        hs[0].step()
        # same inputs, flag set with rho = 1
        h = hs[1]
        p_flags = co2.CO2_FLAG_ANCHOR_PULL
        cur, nxt = h.own[h.t % 2], h.own[(h.t + 1) % 2]
        h._fill_drift(nxt, 100)
        torch.add(h.a, nxt, out=h.x)
        if h.t >= 1:
            for k, pb in enumerate(h.peers):
                h._fill_drift(pb, 200 + k)
        p = co2.make_params(h.seg, 3, 1.0, 0.9, 0.01, 1.0, 4, h.t, p_flags, pull_rho=1.0)
        co2.co2_outer_step(p, h.x, h.a, h.a, h.m, [cur] + h.peers, nxt, None, h.lam, h.ws)
        h.t += 1
        for name in ("x", "a", "m"):
            assert torch.equal(getattr(hs[0], name), getattr(h, name)), name


def test_variants_at_gpt2_small_size(dev):
    """Full-size buffers (124M parameters, K=8); oracle on a sample of whole segments
    that includes the token embedding (38.6M elements, rescaled) and LayerNorm vectors."""
    cfg = co2_inputs.CONFIGS["gpt2s"]
    table = co2_inputs.config_table(cfg)
    sample = [0, 1, 2, 3, 4, 5, 6, 7, 140, 141, 146, 147]
    h = OuterStepHarness(table, HP(K=cfg.K, beta=0.9, phi=0.2, c=1.0), dev, seed=55, sample=sample,
                         momentum_std=1e-3, use_first_step_norm=True, nonstale=True, norm_clip=True,
                         pull_rho=0.5)
    steps(h, 4, carried_from=1)
    assert np.any(h.last["scale"] < 1.0) and np.any(h.last["scale"] == 1.0)


def test_variant_flags_are_rejected_where_they_do_not_apply(dev):
    seg = co2.SegmentTable([0, 512], dev)
    f32 = dict(dtype=torch.float32, device=dev)
    a, m, x, d0, d1, dout = (torch.zeros(512, **f32) for _ in range(6))
    ws = torch.empty(co2.workspace_bytes(512, 1, 2), dtype=torch.uint8, device=dev)
    clipped = torch.zeros(1, dtype=torch.int64, device=dev)
    # split form has no local parameters: neither the current-round mean nor the pull can be formed
    for fl in (co2.CO2_FLAG_CURRENT_ROUND, co2.CO2_FLAG_ANCHOR_PULL):
        p = co2.make_params(seg, 2, 1.0, 0.9, 1.0, 0.0, 4, 1, fl, pull_rho=0.5)
        assert co2.co2_outer_step(p, None, a, torch.empty_like(a), m, [d0, d1], None, None, None, ws,
                                  check=False) == co2.CO2_EINVAL
    p = co2.make_params(seg, 2, 1.0, 0.9, 1.0, 0.0, 4, 1, co2.CO2_FLAG_NORM_CLIP, clipped_out=clipped)
    assert co2.co2_outer_step(p, x, a, a, m, [d0, d1], dout, None, None, ws, check=False) == co2.CO2_EINVAL
    # reduced-precision entry points take no variant flags
    h16 = torch.zeros(512, dtype=torch.bfloat16, device=dev)
    p = co2.make_params(seg, 2, 1.0, 0.9, 1.0, 0.0, 4, 1, co2.CO2_FLAG_NORM_CLIP)
    assert co2.co2_outer_step_bf16(p, x, a, a, m, [h16, h16.clone()], h16.clone(), None, None, ws,
                                   check=False) == co2.CO2_EINVAL


# ------------------------------------------------------------------ binary16 transport
@pytest.mark.parametrize("mode", ["two_pass", "carried", "split"])
def test_f16_deltas_multi_step(dev, mode):
    table = co2_inputs.gpt_table(layers=3, d=97, ffn=385, vocab=3001, ctx=63)
    h = OuterStepHarness(table, HP(K=8, beta=0.95, phi=2e-3, c=1.0), dev, seed=56,
                         momentum_std=0.0, drift="student_t", truth=True, transport="f16")
    for t in range(6):
        flags = co2.CO2_FLAG_CARRIED_NORMS if (mode == "carried" and t >= 1) else 0
        print(f"  f16 {mode} t={t}", flush=True)
        h.step(flags=flags, split=(mode == "split"))
    assert h.last["nclipped"] > 0 and np.any(h.last["lam"] > 1.0)


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
@pytest.mark.parametrize("K", [1, 3, 16])
def test_f16_deltas_edge_shapes(dev, name, K):
    # drift scale 1e-5: most pseudo-gradient coordinates land in binary16's subnormal range
    h = OuterStepHarness(EDGE_TABLES[name], HP(K=K, beta=0.8, phi=0.01, c=1.0, tau=3), dev,
                         seed=57, momentum_std=0.02, truth=True, transport="f16", drift_scale=1e-5)
    for _ in range(3):
        h.step()


def test_f16_deltas_7b_shard_every_element(dev):
    """One 7B shard (421M parameters, K=8) with binary16 transport: every element of
    every output, three rounds, the last in the carried form."""
    cfg = co2_inputs.CONFIGS["7b_shard"]
    table = co2_inputs.config_table(cfg, rank=1)
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=cfg.phi, c=cfg.c, tau=cfg.tau)
    h = StreamedOuterStepHarness(table, hp, dev, seed=cfg.seed, drift_scale=cfg.drift_scale,
                                 momentum_std=cfg.momentum_std, start_step=1, transport="f16",
                                 chunk_elems=1 << 25)
    for i in range(3):
        res = h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if i >= 2 else 0)
        print(f"  7b shard f16 step {h.t - 1}: {res}", flush=True)
    assert res["lam_max"] > 1.0


def test_variants_7b_shard_every_element(dev):
    """All three switches together on one 7B shard at its real size (421M parameters,
    K=8, partial first/last tensors): every element of params, anchor, momentum and
    delta_out and every Lambda against the oracle's own full state, four rounds from
    round 0, carried sums from the second; the pulled local parameters carry over."""
    cfg = co2_inputs.CONFIGS["7b_shard"]
    table = co2_inputs.config_table(cfg, rank=1)
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=0.5, c=cfg.c, tau=cfg.tau)
    h = StreamedOuterStepHarness(table, hp, dev, seed=61, drift_scale=cfg.drift_scale,
                                 momentum_std=cfg.momentum_std, start_step=0, chunk_elems=1 << 25,
                                 nonstale=True, norm_clip=True, pull_rho=0.5, use_first_step_norm=True)
    assert h.ch.n == 421_150_976
    rescaled = []
    for i in range(4):
        res = h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if i >= 1 else 0)
        print(f"  7b shard variants round {h.t - 1}: {res}", flush=True)
        rescaled.append(res["rescaled_segments"])
    assert res["lam_max"] > 1.0
    assert 0 < max(rescaled) < len(table) - 1, "the rescale should bite on some segments only"


@pytest.mark.parametrize("variant", ["anchor_pull", "norm_clip"])
def test_single_variant_gpt2_small_every_element(dev, variant):
    """One switch at a time on the GPT-2-small table, stale order, every element, 3 rounds."""
    cfg = co2_inputs.CONFIGS["gpt2s"]
    table = co2_inputs.config_table(cfg)
    hp = HP(K=cfg.K, alpha=cfg.alpha, beta=cfg.beta, phi=0.05, c=cfg.c, tau=cfg.tau)
    h = StreamedOuterStepHarness(table, hp, dev, seed=62, drift_scale=cfg.drift_scale,
                                 momentum_std=1e-3, start_step=1, chunk_elems=1 << 24, **VARIANTS[variant])
    for i in range(3):
        res = h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if i >= 1 else 0)
        print(f"  gpt2s {variant} round {h.t - 1}: {res}", flush=True)
    assert res["lam_max"] > 1.0
