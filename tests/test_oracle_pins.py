"""Pins for the CPU oracle: things the paper and the mathematics fix, none of
which is the oracle's own formula retyped.

  P0  hand-expanded four-coordinate example (tests/golden), all readings of Eq. 3
  P1  K=1, c=0, no clipping  == library momentum SGD on the pseudo-gradient
      (the SlowMo form the paper starts from in Section 3.2); beta=0, alpha=1
      == plain parameter averaging (Section 3.1, Local-SGD)
  P2  K identical workers == one worker
  P3  mean_k(a - x_k) == a - mean_k x_k  (appendix, local update rule summed)
  P4  |Clip| <= phi, |x' - a| <= alpha*phi, clipped count
  P5  Lambda >= 1, == 1 for c=0 or m=0, affine in c and alpha, inverse in T
  P6  alpha*sqrt(M2) at round t == ||anchor_t - anchor_{t-1}|| from saved anchors
  P7  geometric closed form of the momentum; heavy-ball recursion (appendix)
  P8  first round == general update with m=0 and zero deltas
  P10 AdamW == library AdamW; lr=0 leaves params alone
"""
import json
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "outer_step_worked_example.json")
INF = float("inf")


def f32(a):
    """Fresh contiguous fp32 copy (never a view of the argument)."""
    return np.array(a, dtype=np.float32, copy=True, order="C")


def f64(a):
    """Fresh contiguous fp64 copy (never a view of the argument)."""
    return np.array(a, dtype=np.float64, copy=True, order="C")


def rng_state(seed, n, K, m_std=0.02, drift=1e-3):
    r = np.random.default_rng(seed)
    a = f32(r.normal(0, 0.02, n))
    x = f32(a + r.normal(0, drift, n))
    m = f32(r.normal(0, m_std, n))
    d = [f32(r.normal(0, drift, n)) for _ in range(K)]
    return a, x, m, d


# ---------------------------------------------------------------- P0
with open(GOLDEN) as fh:
    _G = json.load(fh)


@pytest.mark.parametrize("case", _G["cases"], ids=[c["name"] for c in _G["cases"]])
@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_p0_hand_expanded_example(oracle, case, prec):
    c = _G["common"]
    conv = f32 if prec == "f32" else f64
    tol = 2e-7 if prec == "f32" else 2e-9   # fixture is rounded at the 9th digit
    a, x, m = conv(c["a"]), conv(c["x"]), conv(c["m"])
    d = [conv(c["d0"]), conv(c["d1"])]
    fs = None if case["first_step_norm"] is None else conv(case["first_step_norm"])
    fn = oracle.outer_step_f32 if prec == "f32" else oracle.outer_step_f64
    out = fn(seg_off=case["seg_off"], alpha=c["alpha"], beta=c["beta"], phi=c["phi"],
             c=c["c"], tau=c["tau"], step=c["step"], x=x, a=a, m=m, deltas=d,
             first_step_norm=fs)
    # a - x cancels: accurate to the rounding of its operands (|a|, |x| <= 2.1)
    np.testing.assert_allclose(out["dout"], c["dout"], rtol=0, atol=2.1 * tol)
    np.testing.assert_allclose(out["lam"], case["lambda"], rtol=tol)
    np.testing.assert_allclose(m, case["m_new"], rtol=tol)
    np.testing.assert_allclose(x, case["x_new"], rtol=tol)
    np.testing.assert_allclose(a, case["x_new"], rtol=tol)   # anchor <- x_{t+1,0}
    if prec == "f32":
        assert out["nclipped"] == case["nclipped"]


def test_p0_separate_anchor_out_and_split_form(oracle):
    """anchor_out != anchor leaves the anchor alone; x=None skips dout/params."""
    c, case = _G["common"], _G["cases"][0]
    a, m = f32(c["a"]), f32(c["m"])
    a_out = np.zeros(4, np.float32)
    out = oracle.outer_step_f32(seg_off=case["seg_off"], alpha=c["alpha"], beta=c["beta"],
                                phi=c["phi"], c=c["c"], tau=c["tau"], step=1, x=None, a=a,
                                a_out=a_out, m=m, deltas=[f32(c["d0"]), f32(c["d1"])],
                                first_step_norm=f32(case["first_step_norm"]))
    assert out["dout"] is None
    np.testing.assert_array_equal(a, f32(c["a"]))
    np.testing.assert_allclose(a_out, case["x_new"], rtol=2e-7)
    np.testing.assert_allclose(m, case["m_new"], rtol=2e-7)


# ---------------------------------------------------------------- P1
def test_p1_reduces_to_library_momentum_sgd(oracle):
    n, alpha, beta, T = 257, 0.7, 0.9, 5
    r = np.random.default_rng(1)
    a0 = r.normal(0, 0.02, n)
    grads = [r.normal(0, 1e-3, n) for _ in range(T)]

    p = torch.nn.Parameter(torch.tensor(a0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=alpha, momentum=beta, dampening=0.0, nesterov=False)

    a, m = f64(a0), np.zeros(n)
    for t in range(T):
        p.grad = torch.tensor(grads[t], dtype=torch.float64)
        opt.step()
        x = f64(a - 0.5 * grads[t])            # any local params: only dout depends on them
        oracle.outer_step_f64(seg_off=[0, 100, n], alpha=alpha, beta=beta, phi=INF, c=0.0,
                              tau=3, step=t + 1, x=x, a=a, m=m, deltas=[f64(grads[t])])
        np.testing.assert_allclose(a, p.detach().numpy(), rtol=1e-13, atol=1e-16)
        np.testing.assert_array_equal(x, a)

    # fp32 evaluation follows the same trajectory to fp32 accuracy
    a32, m32 = f32(a0), np.zeros(n, np.float32)
    for t in range(T):
        oracle.outer_step_f32(seg_off=[0, 100, n], alpha=alpha, beta=beta, phi=INF, c=0.0,
                              tau=3, step=t + 1, x=f32(a32), a=a32, m=m32,
                              deltas=[f32(grads[t])])
    np.testing.assert_allclose(a32, a, rtol=0, atol=2e-7 * T)


def test_p1_plain_parameter_averaging(oracle):
    n, K = 131, 5
    r = np.random.default_rng(2)
    a0 = r.normal(0, 0.02, n)
    xs = [a0 + r.normal(0, 1e-3, n) for _ in range(K)]
    a, m = f64(a0), f64(r.normal(0, 1, n))       # beta = 0 must erase old momentum
    oracle.outer_step_f64(seg_off=[0, n], alpha=1.0, beta=0.0, phi=INF, c=0.0, tau=1, step=1,
                          x=f64(xs[0]), a=a, m=m, deltas=[f64(a0 - xk) for xk in xs])
    np.testing.assert_allclose(a, np.mean(xs, axis=0), rtol=1e-12)


# ---------------------------------------------------------------- P2
@pytest.mark.parametrize("K", [2, 4, 8, 16])
def test_p2_identical_workers_equal_single_worker(oracle, K):
    n = 1000
    a, x, m, d = rng_state(3, n, 1)
    kw = dict(seg_off=[0, 10, 500, n], alpha=1.0, beta=0.9, phi=0.01, c=1.0, tau=4, step=2)
    a1, x1, m1 = a.copy(), x.copy(), m.copy()
    o1 = oracle.outer_step_f32(x=x1, a=a1, m=m1, deltas=[d[0]], **kw)
    aK, xK, mK = a.copy(), x.copy(), m.copy()
    oK = oracle.outer_step_f32(x=xK, a=aK, m=mK, deltas=[d[0]] * K, **kw)
    np.testing.assert_array_equal(o1["lam"], oK["lam"])
    if K == 2:
        # d + d and the product with 1/2 are exact, so bits agree
        np.testing.assert_array_equal(m1, mK)
        np.testing.assert_array_equal(a1, aK)
    else:
        # the left-to-right sum d+d+...+d rounds at 3d, 5d, ...: each of the
        # K-1 additions is off by at most half an ulp of the running sum; the
        # final sum beta*m + dbar/Lambda may then round one ulp of m' apart
        bound = K * 2.0 ** -24 * np.abs(d[0].astype(np.float64)) + 1e-45
        assert np.all(np.abs(m1.astype(np.float64) - mK)
                      <= bound + 2.0 ** -23 * np.abs(m1.astype(np.float64)))
        assert np.all(np.abs(a1.astype(np.float64) - aK)
                      <= bound + 2.0 ** -23 * np.abs(m1.astype(np.float64))
                      + 2.0 ** -23 * np.abs(a1.astype(np.float64)))


def test_p2_identical_workers_non_power_of_two(oracle):
    n = 1000
    a, x, m, d = rng_state(4, n, 1)
    kw = dict(seg_off=[0, n], alpha=1.0, beta=0.9, phi=INF, c=1.0, tau=4, step=2)
    a1, m1 = f64(a), f64(m)
    oracle.outer_step_f64(x=f64(x), a=a1, m=m1, deltas=[f64(d[0])], **kw)
    a3, m3 = f64(a), f64(m)
    oracle.outer_step_f64(x=f64(x), a=a3, m=m3, deltas=[f64(d[0])] * 3, **kw)
    np.testing.assert_allclose(m3, m1, rtol=1e-14, atol=1e-18)
    np.testing.assert_allclose(a3, a1, rtol=1e-14)


# ---------------------------------------------------------------- P3
def test_p3_mean_of_deltas_is_delta_of_mean(oracle):
    n, K = 300, 8
    r = np.random.default_rng(5)
    a0 = r.normal(0, 0.02, n)
    xs = [a0 + r.normal(0, 1e-3, n) for _ in range(K)]
    m0 = r.normal(0, 0.01, n)
    kw = dict(seg_off=[0, 7, n], alpha=0.9, beta=0.8, phi=INF, c=1.0, tau=2, step=1,
              first_step_norm=f64([0.01, 0.02]))
    a1, m1 = f64(a0), f64(m0)
    oracle.outer_step_f64(x=f64(xs[0]), a=a1, m=m1, deltas=[f64(a0 - xk) for xk in xs], **kw)
    a2, m2 = f64(a0), f64(m0)
    oracle.outer_step_f64(x=f64(xs[0]), a=a2, m=m2,
                          deltas=[f64(a0 - np.mean(xs, axis=0))], **kw)
    np.testing.assert_allclose(m1, m2, rtol=1e-11, atol=1e-16)
    np.testing.assert_allclose(a1, a2, rtol=1e-12)


# ---------------------------------------------------------------- P4
@pytest.mark.parametrize("phi", [1e-3, 5e-3, 1.0])
def test_p4_clipping_bounds_and_count(oracle, phi):
    n, alpha = 5000, 0.75
    a, x, m, d = rng_state(6, n, 4, m_std=0.02)
    a_old, m_old = a.copy(), m.copy()
    out = oracle.outer_step_f32(seg_off=[0, 1234, n], alpha=alpha, beta=0.9, phi=phi, c=0.5,
                                tau=4, step=1, x=x, a=a, m=m, deltas=d)
    moved = np.abs(a.astype(np.float64) - a_old.astype(np.float64))
    assert moved.max() <= alpha * phi * (1 + 2.0 ** -22) + np.abs(a_old).max() * 2.0 ** -23
    assert out["nclipped"] == int(np.count_nonzero(np.abs(m) > np.float32(phi)))
    if phi < 0.01:
        assert out["nclipped"] > n // 2       # the clamp branch is really exercised
        clipped = np.abs(m) > np.float32(phi)
        # clipped coordinates move by exactly alpha*phi (up to rounding of x)
        np.testing.assert_allclose(moved[clipped], alpha * phi, rtol=1e-4)
        # and in the direction opposite to the momentum's sign
        assert np.all(np.sign(a_old[clipped] - a[clipped]) == np.sign(m[clipped]))
    np.testing.assert_array_equal(x, a)
    assert not np.array_equal(m, m_old)


# ---------------------------------------------------------------- P5
def test_p5_lambda_properties(oracle):
    n = 4096
    a, x, m, d = rng_state(7, n, 2)
    seg = [0, 100, 100, 3000, n]              # includes an empty segment
    base = dict(seg_off=seg, beta=0.9, phi=1.0, tau=4, step=1)

    def lam(c=1.0, alpha=1.0, mm=m, fs=None, tau=4):
        kw = dict(base); kw["tau"] = tau
        o = oracle.outer_step_f32(alpha=alpha, c=c, x=x.copy(), a=a.copy(), m=mm.copy(),
                                  deltas=d, first_step_norm=fs, **kw)
        return o["lam"].astype(np.float64)

    L1 = lam()
    assert np.all(L1 >= 1.0) and L1[1] == 1.0          # empty segment: T = 0 -> 1
    assert np.all(L1[[0, 2, 3]] > 1.0)
    assert np.all(lam(c=0.0) == 1.0)
    assert np.all(lam(mm=np.zeros_like(m)) == 1.0)
    np.testing.assert_allclose(lam(c=2.0) - 1, 2 * (L1 - 1), rtol=1e-6)
    np.testing.assert_allclose(lam(alpha=0.5) - 1, 0.5 * (L1 - 1), rtol=1e-6)
    fs = f32([0.01, 0.01, 0.02, 0.04])
    Lf = lam(fs=fs)
    np.testing.assert_allclose(lam(fs=f32(2 * fs)) - 1, (Lf - 1) / 2, rtol=1e-6)
    np.testing.assert_allclose(lam(fs=fs, tau=8) - 1, (Lf - 1) / 2, rtol=1e-6)
    # against the definition: numerator is the norm of the clipped old momentum
    num = np.sqrt(np.add.reduceat(np.clip(m.astype(np.float64), -1, 1) ** 2, [0, 100, 3000]))
    np.testing.assert_allclose(Lf[[0, 2, 3]], num / (4 * fs[[0, 2, 3]].astype(np.float64)) + 1,
                               rtol=1e-6)


# ---------------------------------------------------------------- P6
def test_p6_numerator_equals_anchor_displacement(oracle):
    n, K, alpha, phi = 6000, 3, 0.8, 2e-3
    seg = [0, 1000, 2500, n]
    r = np.random.default_rng(8)
    a = f64(r.normal(0, 0.02, n))
    m = np.zeros(n)
    anchors = [a.copy()]
    for t in range(1, 6):
        d = [f64(r.normal(0, 1e-3, n)) for _ in range(K)]
        prev_m = m.copy()
        out = oracle.outer_step_f32(seg_off=seg, alpha=alpha, beta=0.9, phi=phi, c=1.0, tau=2,
                                    step=t, x=f32(a), a=(a32 := f32(a)), m=(m32 := f32(m)),
                                    deltas=[f32(v) for v in d])
        # redo in fp64 to carry an accurate trajectory
        oracle.outer_step_f64(seg_off=seg, alpha=alpha, beta=0.9, phi=phi, c=1.0, tau=2,
                              step=t, x=f64(a), a=a, m=m, deltas=d)
        anchors.append(a.copy())
        if t >= 2:
            disp = anchors[t - 1] - anchors[t - 2]      # x_{t,0} - x_{t-1,0} seen at round t
            want = np.sqrt(np.add.reduceat(disp ** 2, seg[:-1]))
            got = alpha * np.sqrt(out["M2"])
            np.testing.assert_allclose(got, want, rtol=1e-5)
            assert np.any(np.abs(prev_m) > phi)          # clipping took part in the identity


# ---------------------------------------------------------------- P7
def test_p7_geometric_momentum_and_heavy_ball(oracle):
    n, alpha, beta, T = 64, 0.3, 0.85, 12
    r = np.random.default_rng(9)
    g = r.normal(0, 1e-3, n)
    a, m = f64(r.normal(0, 0.02, n)), np.zeros(n)
    hist = [a.copy()]
    for t in range(1, T + 1):
        oracle.outer_step_f64(seg_off=[0, n], alpha=alpha, beta=beta, phi=INF, c=0.0, tau=1,
                              step=t, x=f64(a), a=a, m=m, deltas=[f64(g)])
        hist.append(a.copy())
        np.testing.assert_allclose(m, g * (1 - beta ** t) / (1 - beta), rtol=1e-12)
    for t in range(1, T):
        lhs = hist[t + 1] - hist[t]
        rhs = beta * (hist[t] - hist[t - 1]) - alpha * g
        np.testing.assert_allclose(lhs, rhs, rtol=1e-9, atol=1e-18)


def test_p7_heavy_ball_with_penalty(oracle):
    """x_{t+1}-x_t = beta (x_t-x_{t-1}) - (alpha/Lambda_t) dbar_t while nothing clips."""
    n, alpha, beta = 500, 0.6, 0.7
    seg = [0, 200, n]
    r = np.random.default_rng(10)
    a, m = f64(r.normal(0, 0.02, n)), np.zeros(n)
    hist = [a.copy()]
    for t in range(1, 7):
        d = [f64(r.normal(0, 1e-3, n)) for _ in range(2)]
        out = oracle.outer_step_f64(seg_off=seg, alpha=alpha, beta=beta, phi=INF, c=1.0,
                                    tau=3, step=t, x=f64(a), a=a, m=m, deltas=d)
        hist.append(a.copy())
        if t >= 2:
            lam = np.repeat(out["lam"], np.diff(seg))
            assert np.all(out["lam"] > 1.0)
            lhs = hist[t] - hist[t - 1]
            rhs = beta * (hist[t - 1] - hist[t - 2]) - alpha / lam * (d[0] + d[1]) / 2
            np.testing.assert_allclose(lhs, rhs, rtol=1e-8, atol=1e-17)


# ---------------------------------------------------------------- P8
def test_p8_first_round(oracle):
    n = 777
    a, x, m, d = rng_state(11, n, 2)
    m[:] = 0
    a0, x0 = a.copy(), x.copy()
    out = oracle.outer_step_f32(seg_off=[0, 5, n], alpha=1.0, beta=0.9, phi=1.0, c=1.0, tau=4,
                                step=0, x=x, a=a, m=m, deltas=None)
    np.testing.assert_array_equal(out["dout"], a0 - x0)
    np.testing.assert_array_equal(x, a0)
    np.testing.assert_array_equal(a, a0)
    assert not m.any() and np.all(out["lam"] == 1.0)
    # the general update with m = 0 and zero deltas lands on the same state
    a2, x2, m2 = a0.copy(), x0.copy(), np.zeros(n, np.float32)
    z = [np.zeros(n, np.float32)] * 2
    out2 = oracle.outer_step_f32(seg_off=[0, 5, n], alpha=1.0, beta=0.9, phi=1.0, c=1.0,
                                 tau=4, step=1, x=x2, a=a2, m=m2, deltas=z)
    np.testing.assert_array_equal(out2["dout"], out["dout"])
    np.testing.assert_array_equal(x2, a0)
    np.testing.assert_array_equal(a2, a0)
    assert not m2.any()


# ---------------------------------------------------------------- norms
def test_sqnorms_against_numpy(oracle):
    r = np.random.default_rng(12)
    buf = f32(r.normal(0, 1, 10007))
    seg = [0, 1, 1, 4096, 9000, 10007]
    got = oracle.sqnorms(buf, seg)
    b64 = buf.astype(np.float64)
    want = [float(np.dot(b64[lo:hi], b64[lo:hi])) for lo, hi in zip(seg, seg[1:])]
    np.testing.assert_allclose(got, want, rtol=1e-13)
    gotc = oracle.sqnorms(buf, seg, phi=0.5)
    c64 = np.clip(b64, -0.5, 0.5)
    wantc = [float(np.dot(c64[lo:hi], c64[lo:hi])) for lo, hi in zip(seg, seg[1:])]
    np.testing.assert_allclose(gotc, wantc, rtol=1e-13)


def test_f32_evaluation_tracks_f64_truth(oracle):
    """The fp32-ordered oracle stays within fp32 rounding of the fp64 one,
    measured against the magnitude of the operands of each sum."""
    n, K = 20000, 8
    a, x, m, d = rng_state(13, n, K)
    seg = [0, 3, 4000, 4001, n]
    kw = dict(seg_off=seg, alpha=1.0, beta=0.95, phi=0.02, c=1.0, tau=4, step=1)
    a32, x32, m32 = a.copy(), x.copy(), m.copy()
    o32 = oracle.outer_step_f32(x=x32, a=a32, m=m32, deltas=d, **kw)
    a64, x64, m64 = f64(a), f64(x), f64(m)
    o64 = oracle.outer_step_f64(x=x64, a=a64, m=m64, deltas=[f64(v) for v in d], **kw)
    np.testing.assert_allclose(o32["lam"], o64["lam"], rtol=2e-7)
    lam = np.repeat(o64["lam"], np.diff(seg))
    dbar = np.mean([f64(v) for v in d], axis=0)
    scale_m = np.abs(0.95 * f64(m)) + np.abs(dbar / lam)
    assert np.all(np.abs(m32 - m64) <= 1e-6 * scale_m)
    scale_x = np.abs(f64(a)) + np.abs(np.clip(m64, -0.02, 0.02))
    assert np.all(np.abs(a32 - a64) <= 1e-6 * scale_x)
    assert np.all(np.abs(o32["dout"] - o64["dout"]) <= 1e-7 * (np.abs(f64(a)) + np.abs(f64(x))))


# ---------------------------------------------------------------- P10
def _bf16_bits(v):
    t = torch.tensor(v, dtype=torch.float32).to(torch.bfloat16)
    return t.view(torch.int16).numpy().astype(np.uint16), t.to(torch.float64).numpy()


def test_p10_adamw_against_library(oracle):
    n, steps = 513, 6
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    r = np.random.default_rng(14)
    p0 = r.normal(0, 0.02, n)
    p_t = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.AdamW([p_t], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]),
                            eps=hp["eps"], weight_decay=hp["weight_decay"], amsgrad=False)
    p64, m64, v64 = f64(p0), np.zeros(n), np.zeros(n)
    p32, m32, v32 = f32(p0), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for k in range(1, steps + 1):
        bits, g = _bf16_bits(r.normal(0, 1e-3, n))
        p_t.grad = torch.tensor(g)
        opt.step()
        oracle.adamw_f64(p=p64, grad=f64(g), exp_avg=m64, exp_avg_sq=v64, k=k, **hp)
        np.testing.assert_allclose(p64, p_t.detach().numpy(), rtol=1e-12, atol=1e-15)
        oracle.adamw_f32(p_in=p32, p_out=p32, grad_bf16=bits, exp_avg=m32, exp_avg_sq=v32,
                         k=k, **hp)
        np.testing.assert_allclose(p32, p64, rtol=0, atol=3e-7 * k * (np.abs(p0).max() + 1e-3))
        # exp_avg is a cancelling sum of terms of size ~1e-3: absolute bound
        np.testing.assert_allclose(m32, m64, rtol=0, atol=1e-3 * 1e-6)
        np.testing.assert_allclose(v32, v64, rtol=1e-5, atol=1e-16)


def test_p10_adamw_epilogues_and_lr_zero(oracle):
    n = 1000
    seg = [0, 10, 10, 600, n]
    r = np.random.default_rng(15)
    p0, anchor = f32(r.normal(0, 0.02, n)), f32(r.normal(0, 0.02, n))
    bits, g = _bf16_bits(r.normal(0, 1e-3, n))
    hp = dict(beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    p1 = np.empty_like(p0)
    out = oracle.adamw_f32(p_in=p0, p_out=p1, grad_bf16=bits, exp_avg=np.zeros(n, np.float32),
                           exp_avg_sq=np.zeros(n, np.float32), lr=3e-4, k=1, anchor=anchor,
                           seg_off=seg, want_step_sq=True, **hp)
    np.testing.assert_array_equal(out["dout"], anchor - p1)
    df = (p1 - p0).astype(np.float64)
    want = [float(np.dot(df[lo:hi], df[lo:hi])) for lo, hi in zip(seg, seg[1:])]
    np.testing.assert_allclose(out["step_sq"], want, rtol=1e-13)
    # closed form of the first step from zero state: bias correction cancels the
    # (1-beta) factors, leaving p*(1-lr*wd) - lr*g/(|g|+eps)
    closed = p0.astype(np.float64) * (1 - 3e-4 * 0.1) - 3e-4 * g / (np.abs(g) + 1e-8)
    np.testing.assert_allclose(p1, closed, rtol=0, atol=2e-7 * 0.1)
    p2 = np.empty_like(p0)
    oracle.adamw_f32(p_in=p0, p_out=p2, grad_bf16=bits, exp_avg=np.zeros(n, np.float32),
                     exp_avg_sq=np.zeros(n, np.float32), lr=0.0, k=1, **hp)
    np.testing.assert_array_equal(p2, p0)


# ---------------------------------------------------------------- bf16 transport
def test_bf16_rounding_against_library_cast(oracle):
    """The oracle's fp32->bf16 (nearest, ties to even) against torch's cast, on
    random values, exact ties in both directions, the largest finite values,
    denormals, zeros and infinities."""
    r = np.random.default_rng(20)
    vals = list(r.normal(0, 1e-3, 2000).astype(np.float32)) + list(r.normal(0, 1e3, 500).astype(np.float32))
    bits = np.array([0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0xBF808000, 0xBF818000,
                     0x7F7FFFFF, 0x7F7F8000, 0x7F7F7FFF, 0x00000001, 0x00008000, 0x00018000,
                     0x807FFFFF, 0x00000000, 0x80000000, 0x7F800000, 0xFF800000], dtype=np.uint32)
    vals += list(bits.view(np.float32))
    v = np.array(vals, dtype=np.float32)
    want = torch.tensor(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.f32_to_bf16(v)
    np.testing.assert_array_equal(got, want)
    back = oracle.bf16_to_f32(got)
    np.testing.assert_array_equal(back, torch.tensor(v).to(torch.bfloat16).to(torch.float32).numpy())
    nan = oracle.f32_to_bf16(np.array([np.nan], np.float32))
    assert np.isnan(oracle.bf16_to_f32(nan)[0])


@pytest.mark.parametrize("fsn", [False, True])
def test_bf16_step_equals_f32_step_on_widened_inputs(oracle, fsn):
    """With bf16 buffers the update is the fp32 update applied to the widened
    deltas (bit for bit), and delta_out is the fp32 delta rounded once."""
    n, K = 3000, 5
    seg = [0, 7, 7, 1500, n]
    a, x, m, d = rng_state(21, n, K)
    to_bits = lambda v: torch.tensor(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)  # noqa: E731
    widen = lambda b: torch.tensor(b.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()  # noqa: E731
    d_bits = [to_bits(v) for v in d]
    d_wide = [widen(b) for b in d_bits]
    fs = f32([0.01, 0.02, 0.03, 0.04]) if fsn else None
    kw = dict(seg_off=seg, alpha=0.9, beta=0.9, phi=5e-3, c=1.0, tau=3, first_step_norm=fs)
    for step in (0, 1):
        a1, x1, m1 = a.copy(), x.copy(), m.copy()
        o1 = oracle.outer_step_f32(x=x1, a=a1, m=m1, deltas=d_wide if step else None, step=step, **kw)
        a2, x2, m2 = a.copy(), x.copy(), m.copy()
        o2 = oracle.outer_step_bf16(x=x2, a=a2, m=m2, deltas=d_bits if step else None, step=step, **kw)
        np.testing.assert_array_equal(a1, a2)
        np.testing.assert_array_equal(x1, x2)
        np.testing.assert_array_equal(m1, m2)
        np.testing.assert_array_equal(o1["lam"], o2["lam"])
        assert o1["nclipped"] == o2["nclipped"]
        np.testing.assert_array_equal(o2["dout"], to_bits(o1["dout"]))


# ---------------------------------------------------------------- binary16 transport
def test_f16_rounding_against_library_cast(oracle):
    """The oracle's fp32->binary16 (nearest, ties to even, gradual underflow, overflow
    to infinity) against numpy's cast: random values over the normal and subnormal
    ranges, exact ties, the overflow boundary, zeros and infinities; and every one of
    the 65536 bit patterns back to fp32."""
    r = np.random.default_rng(22)
    vals = (list(r.normal(0, 1e-3, 2000)) + list(r.normal(0, 1.0, 500)) + list(r.normal(0, 1e-6, 2000))
            + list(r.normal(0, 3e-8, 500)) + list(r.normal(0, 3e4, 500)))
    vals += [0.0, -0.0, 65504.0, 65519.996, 65520.0, 65536.0, -65520.0, 1e9, -1e9, np.inf, -np.inf,
             2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * (1 + 2.0 ** -20), 3 * 2.0 ** -25, 2.0 ** -14,
             2.0 ** -14 * (1 - 2.0 ** -11), 2.0 ** -14 * (1 - 2.0 ** -12), 1 + 2.0 ** -11,
             1 + 3 * 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -20, -(1 + 2.0 ** -11)]
    v = np.array(vals, dtype=np.float32)
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = oracle.f32_to_f16(v)
    np.testing.assert_array_equal(got, want)
    every = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    back = oracle.f16_to_f32(every)
    lib = every.view(np.float16).astype(np.float32)
    both_nan = np.isnan(back) & np.isnan(lib)
    np.testing.assert_array_equal(back[~both_nan], lib[~both_nan])
    assert np.array_equal(np.isnan(back), np.isnan(lib))
    nan = oracle.f32_to_f16(np.array([np.nan], np.float32))
    assert np.isnan(oracle.f16_to_f32(nan)[0])


@pytest.mark.parametrize("fsn", [False, True])
def test_f16_step_equals_f32_step_on_widened_inputs(oracle, fsn):
    """With binary16 buffers the update is the fp32 update applied to the widened
    deltas (bit for bit), and delta_out is the fp32 delta rounded once."""
    n, K = 3000, 5
    seg = [0, 7, 7, 1500, n]
    a, x, m, d = rng_state(23, n, K)
    d[1][:50] *= 1e-4                                         # reach the subnormal range
    to_bits = lambda v: np.asarray(v, np.float32).astype(np.float16).view(np.uint16)  # noqa: E731
    widen = lambda b: b.view(np.float16).astype(np.float32)  # noqa: E731
    d_bits = [to_bits(v) for v in d]
    d_wide = [widen(b) for b in d_bits]
    fs = f32([0.01, 0.02, 0.03, 0.04]) if fsn else None
    kw = dict(seg_off=seg, alpha=0.9, beta=0.9, phi=5e-3, c=1.0, tau=3, first_step_norm=fs)
    for step in (0, 1):
        a1, x1, m1 = a.copy(), x.copy(), m.copy()
        o1 = oracle.outer_step_f32(x=x1, a=a1, m=m1, deltas=d_wide if step else None, step=step, **kw)
        a2, x2, m2 = a.copy(), x.copy(), m.copy()
        o2 = oracle.outer_step_f16(x=x2, a=a2, m=m2, deltas=d_bits if step else None, step=step, **kw)
        np.testing.assert_array_equal(a1, a2)
        np.testing.assert_array_equal(x1, x2)
        np.testing.assert_array_equal(m1, m2)
        np.testing.assert_array_equal(o1["lam"], o2["lam"])
        assert o1["nclipped"] == o2["nclipped"]
        np.testing.assert_array_equal(o2["dout"], to_bits(o1["dout"]))


# ---------------------------------------------------------------- variants of the outer rule
# V0 hand-expanded example per switch (tests/golden)
# V1 every switch off == outer_step_f32, bit for bit
# V2 current-round mean: library momentum SGD from round 0; beta=0, alpha=1 == average of the
#    workers' CURRENT parameters (Section 3.1's Local-SGD line)
# V3 anchor pull: only the local parameters depend on rho; library lerp; rho=1/2 is the midpoint
# V4 norm rescale: step norm <= alpha*phi; untouched segments == no clipping; library
#    clip_grad_norm_; numerator of Eq. 3 == measured anchor displacement
VGOLDEN = os.path.join(os.path.dirname(__file__), "golden", "outer_step_variants_worked_example.json")
with open(VGOLDEN) as fh:
    _V = json.load(fh)


@pytest.mark.parametrize("case", _V["cases"], ids=[c["name"] for c in _V["cases"]])
def test_v0_hand_expanded_variants(oracle, case):
    c = _V["common"]
    tol = 2e-7
    a, x, m = f32(c["a"]), f32(c["x"]), f32(case["m"])
    d0 = None if case["nonstale"] else f32(c["d0"])
    if case["nonstale"]:
        d_unused = f32([9.0, 9.0, 9.0, 9.0])       # must not be read
        deltas = [d_unused, f32(c["d1"])]
    else:
        deltas = [d0, f32(c["d1"])]
    fs = None if case["first_step_norm"] is None else f32(case["first_step_norm"])
    out = oracle.outer_step_variant_f32(
        seg_off=c["seg_off"], alpha=c["alpha"], beta=c["beta"],
        phi=INF if case["phi"] is None else case["phi"], c=case["c"], tau=c["tau"],
        step=case["step"], x=x, a=a, m=m, deltas=deltas, nonstale=case["nonstale"],
        norm_clip=case["norm_clip"], pull_rho=case["pull_rho"], first_step_norm=fs)
    np.testing.assert_allclose(out["dout"], c["dout"], rtol=0, atol=2.1 * tol)
    np.testing.assert_allclose(out["lam"], case["lambda"], rtol=tol)
    np.testing.assert_allclose(out["scale"], case["scale"], rtol=tol)
    # in the current-round order a - x (a cancelling difference of values up to 2.1) enters m
    np.testing.assert_allclose(m, case["m_new"], rtol=tol, atol=2.1 * tol if case["nonstale"] else 0)
    np.testing.assert_allclose(a, case["anchor_new"], rtol=0, atol=2.1 * tol)
    np.testing.assert_allclose(x, case["params_new"], rtol=0, atol=2.1 * tol)
    assert out["nclipped"] == case["nclipped"]


@pytest.mark.parametrize("use_fsn", [False, True])
def test_v1_all_switches_off_is_the_base_update(oracle, use_fsn):
    n, K = 3001, 5
    table = [0, 0, 17, 1000, 1000, 2500, n]
    a, x, m, d = rng_state(31, n, K)
    fs = f32(np.abs(np.random.default_rng(5).normal(1e-3, 3e-4, len(table) - 1))) if use_fsn else None
    kw = dict(seg_off=table, alpha=0.8, beta=0.9, phi=0.015, c=1.0, tau=3, first_step_norm=fs)
    a1, x1, m1 = a.copy(), x.copy(), m.copy()
    a2, x2, m2 = a.copy(), x.copy(), m.copy()
    for step in (0, 1, 2):
        o1 = oracle.outer_step_f32(x=x1, a=a1, m=m1, deltas=d if step else None, step=step, **kw)
        o2 = oracle.outer_step_variant_f32(x=x2, a=a2, m=m2, deltas=d if step else None, step=step, **kw)
        for u, v in ((a1, a2), (x1, x2), (m1, m2), (o1["dout"], o2["dout"]), (o1["lam"], o2["lam"])):
            np.testing.assert_array_equal(u, v)
        assert o1["nclipped"] == o2["nclipped"] and np.all(o2["scale"] == 1.0)
        x1 += f32(np.random.default_rng(step).normal(0, 1e-3, n)); x2[:] = x1
    # split form too
    a3 = np.empty_like(a1)
    a4 = np.empty_like(a1)
    m3, m4 = m1.copy(), m1.copy()
    oracle.outer_step_f32(x=None, a=a1, a_out=a3, m=m3, deltas=d, step=3, **kw)
    oracle.outer_step_variant_f32(x=None, a=a2, a_out=a4, m=m4, deltas=d, step=3, **kw)
    np.testing.assert_array_equal(a3, a4)
    np.testing.assert_array_equal(m3, m4)


def test_v2_current_round_mean_is_library_momentum_sgd_from_round_zero(oracle):
    """Section 3.2's recursion before the staleness: with the current round's
    pseudo-gradients, no penalty and no clipping the anchor follows the library's
    momentum SGD on the mean pseudo-gradient, starting at round 0."""
    n, K, alpha, beta, T = 211, 4, 0.6, 0.8, 5
    r = np.random.default_rng(7)
    a0 = f32(r.normal(0, 0.02, n))
    p = torch.nn.Parameter(torch.tensor(a0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=alpha, momentum=beta)
    a, m = a0.copy(), np.zeros(n, np.float32)
    for t in range(T):
        xs = [f32(a + r.normal(0, 1e-3, n)) for _ in range(K)]        # the K workers' local parameters
        pg = [a.astype(np.float64) - xk for xk in xs]                 # their pseudo-gradients
        p.grad = torch.tensor(np.mean(pg, axis=0))
        opt.step()
        x = xs[0].copy()
        poison = np.full(n, 1e3, np.float32)                          # d[0] must not be read
        out = oracle.outer_step_variant_f32(
            seg_off=[0, 50, n], alpha=alpha, beta=beta, phi=INF, c=0.0, tau=2, step=t, x=x, a=a, m=m,
            deltas=[poison] + [f32(a_prev - xk) for a_prev, xk in zip([a.copy()] * (K - 1), xs[1:])],
            nonstale=True)
        np.testing.assert_allclose(a, p.detach().numpy(), rtol=0, atol=3e-7 * (t + 1))
        np.testing.assert_array_equal(x, a)
        assert np.all(out["lam"] == 1.0) and out["nclipped"] == 0


def test_v2_current_round_mean_averages_the_workers_parameters(oracle):
    n, K = 97, 6
    r = np.random.default_rng(8)
    a0 = f32(r.normal(0, 0.02, n))
    xs = [f32(a0 + r.normal(0, 1e-3, n)) for _ in range(K)]
    a, m, x = a0.copy(), f32(r.normal(0, 1, n)), xs[0].copy()
    oracle.outer_step_variant_f32(seg_off=[0, n], alpha=1.0, beta=0.0, phi=INF, c=0.0, tau=1, step=0,
                                  x=x, a=a, m=m,
                                  deltas=[np.full(n, 1e3, np.float32)] + [f32(a0 - xk) for xk in xs[1:]],
                                  nonstale=True)                      # d[0] (poisoned) must not be read
    np.testing.assert_allclose(a, np.mean(np.array(xs, dtype=np.float64), axis=0), rtol=0, atol=2e-8)


def test_v2_penalty_in_current_round_order_needs_first_step_norms(oracle):
    a, x, m, d = rng_state(9, 64, 2)
    with pytest.raises(ValueError):
        oracle.outer_step_variant_f32(seg_off=[0, 64], alpha=1.0, beta=0.9, phi=1.0, c=1.0, tau=2,
                                      step=1, x=x, a=a, m=m, deltas=d, nonstale=True)


@pytest.mark.parametrize("rho", [0.5, 0.25, 0.9])
def test_v3_anchor_pull_moves_only_the_local_parameters(oracle, rho):
    n, K = 2000, 3
    table = [0, 300, 300, 1500, n]
    a, x, m, d = rng_state(11, n, K)
    kw = dict(seg_off=table, alpha=0.9, beta=0.9, phi=0.01, c=1.0, tau=4, step=2, deltas=d)
    a1, x1, m1 = a.copy(), x.copy(), m.copy()
    o1 = oracle.outer_step_f32(x=x1, a=a1, m=m1, **kw)
    a2, x2, m2 = a.copy(), x.copy(), m.copy()
    o2 = oracle.outer_step_variant_f32(x=x2, a=a2, m=m2, pull_rho=rho, **kw)
    for u, v in ((a1, a2), (m1, m2), (o1["dout"], o2["dout"]), (o1["lam"], o2["lam"])):
        np.testing.assert_array_equal(u, v)
    # params = x - rho*(x - anchor') : the library's linear interpolation from x towards anchor'
    want = torch.lerp(torch.tensor(x, dtype=torch.float64), torch.tensor(a2, dtype=torch.float64), rho).numpy()
    np.testing.assert_allclose(x2, want, rtol=0, atol=1e-8)      # a few fp32 roundings at |x| ~ 0.05
    if rho == 0.5:
        np.testing.assert_allclose(x2, (x.astype(np.float64) + a2) / 2, rtol=0, atol=1e-8)
    # what is left of the gap to the anchor
    np.testing.assert_allclose(x2.astype(np.float64) - a2, (1 - rho) * (x.astype(np.float64) - a2),
                               rtol=0, atol=1e-8)
    assert not np.array_equal(x2, a2)


def test_v3_pull_needs_local_parameters_and_a_valid_rho(oracle):
    a, x, m, d = rng_state(12, 32, 2)
    for bad in (0.0, -0.5, 1.5, float("nan")):
        with pytest.raises(ValueError):
            oracle.outer_step_variant_f32(seg_off=[0, 32], alpha=1.0, beta=0.9, phi=1.0, c=0.0, tau=2,
                                          step=1, x=x, a=a, m=m, deltas=d, pull_rho=bad)
    with pytest.raises(ValueError):
        oracle.outer_step_variant_f32(seg_off=[0, 32], alpha=1.0, beta=0.9, phi=1.0, c=0.0, tau=2,
                                      step=1, x=None, a=a, a_out=np.empty_like(a), m=m, deltas=d,
                                      pull_rho=0.5)


def test_v4_norm_rescale_against_the_library_and_its_bounds(oracle):
    n, K, alpha, beta = 4000, 4, 0.7, 0.9
    table = [0, 10, 10, 1200, 2600, n]
    phi = 0.25
    a, x, m, d = rng_state(13, n, K, m_std=0.02)
    m[1200:2600] *= 0.01                                   # one segment well inside the threshold
    a0, m0 = a.copy(), m.copy()
    fs = f32([1e-3, 1e-3, 2e-3, 1e-3, 3e-3])
    out = oracle.outer_step_variant_f32(seg_off=table, alpha=alpha, beta=beta, phi=phi, c=1.0, tau=2,
                                        step=2, x=x, a=a, m=m, deltas=d, norm_clip=True,
                                        first_step_norm=fs)
    # same round without any clipping: the momentum is the same, rescaled segments differ in the iterate
    a_u, x_u, m_u = a0.copy(), (a0 + 0).copy(), m0.copy()
    # Lambda must be the norm-rescale one, so feed it through c*ratio by hand: re-run with norm_clip and phi=inf
    free = oracle.outer_step_variant_f32(seg_off=table, alpha=alpha, beta=beta, phi=INF, c=0.0, tau=2,
                                         step=2, x=x_u, a=a_u, m=m_u, deltas=d, norm_clip=True)
    assert np.all(free["scale"] == 1.0) and free["nclipped"] == 0
    rescaled = 0
    for s in range(len(table) - 1):
        lo, hi = table[s], table[s + 1]
        if hi == lo:
            assert out["scale"][s] == 1.0
            continue
        ms = m[lo:hi].astype(np.float64)
        nrm = np.sqrt(np.dot(ms, ms))
        step_norm = np.sqrt(np.sum((a[lo:hi].astype(np.float64) - a0[lo:hi]) ** 2))
        assert step_norm <= alpha * phi * (1 + 1e-6)
        # library: clip_grad_norm_ on a tensor whose .grad is this segment of m_t
        g = torch.nn.Parameter(torch.zeros(hi - lo, dtype=torch.float64))
        g.grad = torch.tensor(ms)
        torch.nn.utils.clip_grad_norm_([g], max_norm=phi)
        want = a0[lo:hi].astype(np.float64) - alpha * g.grad.numpy()
        np.testing.assert_allclose(a[lo:hi], want, rtol=0, atol=1e-5 * alpha * phi)
        if nrm > phi:
            rescaled += hi - lo
            np.testing.assert_allclose(out["scale"][s], phi / nrm, rtol=2e-7)
            np.testing.assert_allclose(step_norm, alpha * phi, rtol=1e-6)
            # direction kept: the step is a multiple of m_t
            ratio = (a0[lo:hi].astype(np.float64) - a[lo:hi]) / ms
            np.testing.assert_allclose(ratio, alpha * phi / nrm, rtol=5e-4)
        else:
            assert out["scale"][s] == 1.0
            np.testing.assert_array_equal(a[lo:hi], f32(a0[lo:hi] - f32(alpha) * m[lo:hi]))
    assert out["nclipped"] == rescaled and 0 < rescaled < n
    np.testing.assert_array_equal(x, a)


def test_v4_norm_rescale_numerator_is_the_measured_anchor_displacement(oracle):
    """Eq. 3's numerator under norm rescale, alpha*min(||m_{t-1}||_s, phi), against
    ||x_{t,0} - x_{t-1,0}||_s measured from saved anchors; Lambda - 1 = c*that/T."""
    n, K, alpha, c, tau = 3000, 3, 0.8, 0.7, 3
    table = [0, 700, 1900, n]
    phi = 0.02
    r = np.random.default_rng(14)
    a = f32(r.normal(0, 0.02, n))
    m = f32(r.normal(0, 4e-4, n))
    m[700:1900] *= 10.0                                     # one segment far beyond the threshold
    anchors = [a.copy()]
    fs_hist = []
    for t in range(1, 5):
        x = f32(a + r.normal(0, 1e-3, n))
        d = [f32(r.normal(0, 1e-3, n)) for _ in range(K)]
        fs = f32(np.abs(r.normal(2e-3, 2e-4, 3)))
        out = oracle.outer_step_variant_f32(seg_off=table, alpha=alpha, beta=0.9, phi=phi, c=c, tau=tau,
                                            step=t, x=x, a=a, m=m, deltas=d, norm_clip=True,
                                            first_step_norm=fs)
        anchors.append(a.copy())
        if t >= 2:
            for s in range(3):
                lo, hi = table[s], table[s + 1]
                moved = np.sqrt(np.sum((anchors[t - 1][lo:hi].astype(np.float64) - anchors[t - 2][lo:hi]) ** 2))
                want = c * moved / (tau * float(fs[s])) + 1.0
                np.testing.assert_allclose(out["lam"][s], want, rtol=2e-6)
            assert np.any(prev_scale < 1.0) and np.any(prev_scale == 1.0)
        prev_scale = out["scale"]
