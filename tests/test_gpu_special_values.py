"""Degenerate VALUES (the degenerate shapes are in test_gpu_outer_step.py): subnormal numbers,
signed zeros, magnitudes whose sum over the workers overflows, infinities and NaN in the
incoming pseudo-gradients, the momentum and the local parameters.  The paper does not say
what the update does with them; what matters here is that the HIP path and the oracle take
the same decisions (Clip(NaN) = phi by Section 3.3's min/max written out, Lambda = 1 over an
infinite denominator, NaN once a segment's denominator is NaN) -- element by element, over
three consecutive rounds so that what one round leaves (an infinite own pseudo-gradient, a NaN
momentum, carried sums that are infinite) is what the next one reads."""
import numpy as np
import pytest
import torch

import paper_2401_16265_amd as co2
from oracle import co2_oracle

pytestmark = pytest.mark.gpu

TABLE = [0, 300, 300, 1000, 1537, 4099]          # an empty segment, boundaries inside tiles, ragged end
N, S, K = TABLE[-1], len(TABLE) - 1, 3
HPK = dict(alpha=0.7, beta=0.9, phi=0.05, c=1.0, tau=4)
NAN, INF = float("nan"), float("inf")


@pytest.fixture()
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def plant(case, rng, x, m, peers, t):
    """Writes the case's special values into round t's inputs (host arrays, in place)."""
    if case == "subnormal":
        # everything the update reads except the anchor sits in fp32's subnormal range
        m *= np.float32(1e-36)
        for p in peers:
            p *= np.float32(1e-37)
    elif case == "signed_zero":
        m[::3] = -0.0
        for p in peers:
            p[::2] = -0.0
        peers[0][::4] = 0.0
    elif case == "overflowing_sum":
        for p in peers:
            p[5::7] = np.float32(3e38)            # own + 3e38 + 3e38 = inf in fp32
            p[6::7] = np.float32(-3e38)
    elif case == "inf_in_peer":
        peers[0][10] = INF                        # segment 0
        peers[1][1200] = -INF                     # segment 3
        peers[0][1300], peers[1][1300] = INF, -INF   # inf - inf = NaN in the mean
    elif case == "nan_in_peer":
        peers[1][700] = NAN                       # segment 2 only
    elif case == "nan_in_momentum" and t == 1:
        m[2000] = NAN                             # segment 4; stays NaN in later rounds by itself
    elif case == "inf_in_params":
        x[20] = INF                               # delta_out = -inf: next round's denominator is infinite
        x[1100] = NAN                             # delta_out = NaN: next round's Lambda of segment 3 is NaN


def same(got, want, what):
    g, w = np.asarray(got), np.asarray(want)
    assert np.array_equal(np.isnan(g), np.isnan(w)), f"{what}: NaN in different places"
    ok = np.isnan(w) | (g == w)
    if not ok.all():
        j = int(np.flatnonzero(~ok)[0])
        raise AssertionError(f"{what}[{j}]: got {g[j]!r} want {w[j]!r} ({int((~ok).sum())} differ)")
    # equal values may still differ in the sign of a zero
    assert np.array_equal(np.signbit(g[~np.isnan(w)]), np.signbit(w[~np.isnan(w)])), f"{what}: sign of zero"


CASES = ["subnormal", "signed_zero", "overflowing_sum", "inf_in_peer", "nan_in_peer", "nan_in_momentum",
         "inf_in_params"]


@pytest.mark.parametrize("form", ["two_pass", "carried"])
@pytest.mark.parametrize("case", CASES)
def test_special_values_fp32(dev, case, form):
    rng = np.random.default_rng(7)
    a = rng.normal(0, 0.02, N).astype(np.float32)
    m = rng.normal(0, 0.02, N).astype(np.float32)
    own = rng.normal(0, 1e-3, N).astype(np.float32)
    seg = co2.SegmentTable(TABLE, dev)
    dv = lambda h: torch.from_numpy(h.copy()).to(dev)
    d_a, d_m = dv(a), dv(m)
    d_own = [torch.empty(N, device=dev), dv(own)]            # ping-pong; round 1 reads [1]
    lam = torch.empty(S, device=dev)
    ws = torch.empty(co2.workspace_bytes(N, S, K), dtype=torch.uint8, device=dev)
    saw_subnormal = False
    for t in (1, 2, 3):
        print(f"case={case} form={form} round={t}", flush=True)
        x = (a + rng.normal(0, 1e-3, N)).astype(np.float32)
        peers = [rng.normal(0, 1e-3, N).astype(np.float32) for _ in range(K - 1)]
        if case == "nan_in_momentum" and t == 1:
            plant(case, rng, x, m, peers, t)
            d_m = dv(m)
        elif case in ("subnormal", "signed_zero") and t == 1:
            plant(case, rng, x, m, peers, t)
            d_m = dv(m)
            if case == "subnormal":
                own *= np.float32(1e-37)                       # round 1's own pseudo-gradient as well
                d_own[1] = dv(own)
        elif case in ("subnormal", "signed_zero"):
            mm = np.zeros(1, np.float32)
            plant(case, rng, x, mm, peers, t)                  # the peers only: m is carried state
        else:
            plant(case, rng, x, m, peers, t)
        d_x, d_peers = dv(x), [dv(p) for p in peers]
        cur, nxt = d_own[t % 2], d_own[(t + 1) % 2]
        flags = co2.CO2_FLAG_CARRIED_NORMS if (form == "carried" and t >= 2) else 0
        p = co2.make_params(seg, K, HPK["alpha"], HPK["beta"], HPK["phi"], HPK["c"], HPK["tau"], t, flags)
        co2.co2_outer_step(p, d_x, d_a, d_a, d_m, [cur] + d_peers, nxt, None, lam, ws)
        torch.cuda.synchronize()
        out = co2_oracle.outer_step_f32(seg_off=np.asarray(TABLE, np.int64), step=t, x=x, a=a, m=m,
                                        deltas=[own] + peers, **HPK)
        own = out["dout"]
        same(d_x.cpu().numpy(), x, "params")
        same(d_a.cpu().numpy(), a, "anchor")
        same(d_m.cpu().numpy(), m, "momentum")
        same(nxt.cpu().numpy(), own, "delta_out")
        g_lam, w_lam = lam.cpu().numpy(), out["lam"]
        assert np.array_equal(np.isnan(g_lam), np.isnan(w_lam)), (g_lam, w_lam)
        fin = ~np.isnan(w_lam)
        np.testing.assert_allclose(g_lam[fin], w_lam[fin], rtol=1e-5, atol=0)
        saw_subnormal |= bool((np.abs(m[m != 0]) < np.finfo(np.float32).tiny).any())
    if case in ("nan_in_peer", "nan_in_momentum", "inf_in_params", "inf_in_peer"):
        assert np.isnan(m).any() or np.isinf(own).any(), "the case did not exercise a non-finite value"
    if case == "subnormal":
        assert saw_subnormal, "no subnormal momentum was produced"


@pytest.mark.parametrize("transport", ["bf16", "f16"])
def test_transport_overflow_and_underflow(dev, transport):
    """16-bit transport: a local drift beyond binary16's range leaves an infinite pseudo-gradient
    pattern, one below its subnormal range a zero; bf16 keeps both.  The patterns written, and
    everything the next rounds make of them, equal the oracle's."""
    rng = np.random.default_rng(11)
    a = rng.normal(0, 0.02, N).astype(np.float32)
    m = rng.normal(0, 0.02, N).astype(np.float32)
    to16 = {"bf16": co2_oracle.f32_to_bf16, "f16": co2_oracle.f32_to_f16}[transport]
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[transport]
    entry = {"bf16": co2.co2_outer_step_bf16, "f16": co2.co2_outer_step_f16}[transport]
    oracle_step = {"bf16": co2_oracle.outer_step_bf16, "f16": co2_oracle.outer_step_f16}[transport]
    own = to16(rng.normal(0, 1e-3, N).astype(np.float32))
    seg = co2.SegmentTable(TABLE, dev)
    dv = lambda h: torch.from_numpy(h.copy()).to(dev)
    bits = lambda h: torch.from_numpy(h.view(np.int16).copy()).to(dev).view(tdt)
    d_a, d_m = dv(a), dv(m)
    d_own = [torch.empty(N, dtype=tdt, device=dev), bits(own)]
    lam = torch.empty(S, device=dev)
    ws = torch.empty(co2.workspace_bytes(N, S, K), dtype=torch.uint8, device=dev)
    for t in (1, 2, 3):
        print(f"transport={transport} round={t}", flush=True)
        drift = rng.normal(0, 1e-3, N).astype(np.float32)
        drift[3::11] = np.float32(1e5) * np.sign(drift[3::11])      # beyond binary16's 65504
        drift[4::11] = np.float32(7e4)                              # rounds to +inf in binary16
        drift[5::11] = np.float32(65519.0)                          # just below the rounding boundary to inf
        drift[6::11] *= np.float32(1e-6)                            # binary16 subnormals and zeros
        x = (a + drift).astype(np.float32)
        peers = [to16(rng.normal(0, 1e-3, N).astype(np.float32)) for _ in range(K - 1)]
        d_x, d_peers = dv(x), [bits(p) for p in peers]
        cur, nxt = d_own[t % 2], d_own[(t + 1) % 2]
        flags = co2.CO2_FLAG_CARRIED_NORMS if t >= 2 else 0
        p = co2.make_params(seg, K, HPK["alpha"], HPK["beta"], HPK["phi"], HPK["c"], HPK["tau"], t, flags)
        entry(p, d_x, d_a, d_a, d_m, [cur] + d_peers, nxt, None, lam, ws)
        torch.cuda.synchronize()
        out = oracle_step(seg_off=np.asarray(TABLE, np.int64), step=t, x=x, a=a, m=m,
                          deltas=[own] + peers, **HPK)
        own = out["dout"]
        got = nxt.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, own), "delta_out patterns differ"
        same(d_x.cpu().numpy(), x, "params")
        same(d_a.cpu().numpy(), a, "anchor")
        same(d_m.cpu().numpy(), m, "momentum")
        np.testing.assert_allclose(lam.cpu().numpy(), out["lam"], rtol=1e-5, atol=0)
    if transport == "f16":
        assert (own == 0x7C00).any() and (own == 0xFC00).any(), "no infinite binary16 pattern was produced"


@pytest.mark.parametrize("case", ["subnormal", "overflowing_sum", "inf_in_peer", "nan_in_peer", "inf_in_params"])
def test_special_values_with_the_variant_switches(dev, case):
    """The same values under current-round mean + anchor pull + clipping by norm rescale: an
    infinite or NaN ||m_t||_s decides the rescale factor of its whole segment, so the decision
    (and the pulled local parameters carried into the next round) must match the oracle's."""
    rng = np.random.default_rng(13)
    a = rng.normal(0, 0.02, N).astype(np.float32)
    m = rng.normal(0, 0.02, N).astype(np.float32)
    x = a.copy()
    fsn = (1e-3 * (1.0 + 0.25 * np.arange(S))).astype(np.float32)
    seg = co2.SegmentTable(TABLE, dev)
    dv = lambda h: torch.from_numpy(h.copy()).to(dev)
    d_a, d_m, d_x, d_fsn = dv(a), dv(m), dv(x), dv(fsn)
    d_out = torch.empty(N, device=dev)
    lam = torch.empty(S, device=dev)
    ws = torch.empty(co2.workspace_bytes(N, S, K), dtype=torch.uint8, device=dev)
    vflags = co2.CO2_FLAG_CURRENT_ROUND | co2.CO2_FLAG_ANCHOR_PULL | co2.CO2_FLAG_NORM_CLIP
    hp = dict(HPK, phi=0.5)
    for t in (0, 1, 2):
        print(f"variants case={case} round={t}", flush=True)
        x = (x + rng.normal(0, 1e-3, N)).astype(np.float32)    # the pulled parameters carry over
        peers = [rng.normal(0, 1e-3, N).astype(np.float32) for _ in range(K - 1)]
        if case == "subnormal":
            if t == 0:
                plant(case, rng, x, m, peers, t)
                d_m = dv(m)
            else:
                plant(case, rng, x, np.zeros(1, np.float32), peers, t)
        else:
            plant(case, rng, x, m, peers, t)
        d_x.copy_(dv(x))
        d_peers = [dv(p) for p in peers]
        flags = vflags | (co2.CO2_FLAG_CARRIED_NORMS if t >= 1 else 0)
        p = co2.make_params(seg, K, hp["alpha"], hp["beta"], hp["phi"], hp["c"], hp["tau"], t, flags,
                            pull_rho=0.5)
        co2.co2_outer_step(p, d_x, d_a, d_a, d_m, [None] + d_peers, d_out, d_fsn, lam, ws)
        torch.cuda.synchronize()
        out = co2_oracle.outer_step_variant_f32(
            seg_off=np.asarray(TABLE, np.int64), step=t, x=x, a=a, m=m,
            deltas=[np.full(N, 1e3, np.float32)] + peers, first_step_norm=fsn, nonstale=True,
            norm_clip=True, pull_rho=0.5, **hp)
        same(d_x.cpu().numpy(), x, "params")
        same(d_a.cpu().numpy(), a, "anchor")
        same(d_m.cpu().numpy(), m, "momentum")
        same(d_out.cpu().numpy(), out["dout"], "delta_out")
        g_lam, w_lam = lam.cpu().numpy(), out["lam"]
        assert np.array_equal(np.isnan(g_lam), np.isnan(w_lam)), (g_lam, w_lam)
        fin = ~np.isnan(w_lam)
        np.testing.assert_allclose(g_lam[fin], w_lam[fin], rtol=1e-5, atol=0)


def test_adamw_special_gradients(dev):
    """The fused AdamW step on bf16 gradients that are zero (second moment stays 0: the update
    divides by eps alone), subnormal, huge (the squared gradient overflows fp32), infinite and
    NaN, and on moments that are already subnormal: every output equals the oracle's."""
    n, table = 4099, [0, 0, 7, 2048, 2048, 4099]
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    rng = np.random.default_rng(17)
    seg = co2.SegmentTable(table, dev)
    o_p = rng.normal(0, 0.02, n).astype(np.float32)
    o_anchor = rng.normal(0, 0.02, n).astype(np.float32)
    o_m1 = (rng.normal(0, 1, n) * 1e-39).astype(np.float32)            # subnormal first moments
    o_v = (np.abs(rng.normal(0, 1, n)) * 1e-41).astype(np.float32)     # subnormal second moments
    dv = lambda h: torch.from_numpy(h.copy()).to(dev)
    p, anchor, m1, v = dv(o_p), dv(o_anchor), dv(o_m1), dv(o_v)
    dout = torch.empty(n, device=dev)
    sq = torch.empty(seg.S, dtype=torch.float64, device=dev)
    ws = torch.empty(co2.workspace_bytes(n, seg.S, 1), dtype=torch.uint8, device=dev)
    for k in range(1, 4):
        print(f"adamw special gradients k={k}", flush=True)
        g = rng.normal(0, 1e-3, n).astype(np.float32)
        g[0::13] = 0.0
        g[1::13] = -0.0
        g[2::13] = 1e-39                     # bf16 subnormal
        g[3::13] = 3e38                      # g*g overflows fp32
        g[4::13] = -3e38
        if k == 2:
            g[5] = INF
            g[2100] = -INF
        if k == 3:
            g[6] = NAN
        gb = co2_oracle.f32_to_bf16(g)
        d_g = torch.from_numpy(gb.view(np.int16).copy()).to(dev).view(torch.bfloat16)
        co2.co2_inner_adamw(n, p, p, d_g, m1, v, adam_step=k, anchor=anchor, delta_out=dout, table=seg,
                            step_sq_out=sq, workspace=ws, **hp)
        torch.cuda.synchronize()
        out = co2_oracle.adamw_f32(p_in=o_p, p_out=o_p, grad_bf16=gb, exp_avg=o_m1, exp_avg_sq=o_v, k=k,
                                   anchor=o_anchor, seg_off=table, want_step_sq=True, **hp)
        same(p.cpu().numpy(), o_p, "params")
        same(m1.cpu().numpy(), o_m1, "exp_avg")
        same(v.cpu().numpy(), o_v, "exp_avg_sq")
        same(dout.cpu().numpy(), out["dout"], "delta_out")
        g_sq, w_sq = sq.cpu().numpy(), out["step_sq"]
        assert np.array_equal(np.isnan(g_sq), np.isnan(w_sq)), (g_sq, w_sq)
        fin = np.isfinite(w_sq)
        assert np.array_equal(g_sq[~fin & ~np.isnan(w_sq)], w_sq[~fin & ~np.isnan(w_sq)])
        np.testing.assert_allclose(g_sq[fin], w_sq[fin], rtol=1e-12, atol=0)
    assert np.isnan(o_p).any() and np.isinf(o_v).any(), "the non-finite gradients were not exercised"
