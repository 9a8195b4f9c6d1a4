"""Pins for the oracle's inner optimizer (AdamW), against things other than itself:
hand-computed one-element steps, closed forms in exact rational arithmetic, and the
float64 AdamW of the PyTorch wheel on the CPU (an independent library routine).

The hyper-parameters deliberately include a large eps and odd betas in several tests, so
that a misplaced eps, swapped betas, a missing bias correction or a coupled (L2) decay
each fail at least one test.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle


def test_one_element_by_hand(paper_hp):
    # theta=1, g=0.1, paper's lr 4e-4 and wd 0.1, beta 0.9/0.999, eps 1e-8.
    # Step 1: m=0.01, v=1e-5, m_hat=0.1, v_hat=0.01, sqrt=0.1
    #   theta1 = 1 - 4e-5 - 4e-4*0.1/(0.1+1e-8) = 0.99956000004 (to 11 places)
    # Step 2 (same g): m_hat, v_hat unchanged -> theta2 = theta1*(1-4e-5) - 3.9999996e-4
    #   = 0.99912001768 (to 11 places)
    hp = paper_hp
    st = oracle.AdamWState([1.0], dtype=np.float64)
    g = np.array([0.1])
    oracle.adamw_step(st, g, hp["inner_lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"])
    assert st.m[0] == pytest.approx(0.01, rel=1e-14)
    assert st.v[0] == pytest.approx(1e-5, rel=1e-12)
    assert st.theta[0] == pytest.approx(0.99956000004, abs=1e-11)
    oracle.adamw_step(st, g, hp["inner_lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"])
    assert st.theta[0] == pytest.approx(0.99912001768, abs=1e-11)
    assert st.t == 2

    # float32 state: same numbers within a couple of float32 ulps of 1.0.
    s32 = oracle.AdamWState([1.0])
    for _ in range(2):
        oracle.adamw_step(s32, g.astype(np.float32), hp["inner_lr"], hp["beta1"], hp["beta2"],
                          hp["eps"], hp["weight_decay"])
    assert abs(float(s32.theta[0]) - 0.99912001768) < 3 * 2.0 ** -24


@pytest.mark.parametrize("g0,eps", [(0.3, 0.05), (-0.02, 0.5), (7.0, 1e-8)])
def test_constant_gradient_closed_form(g0, eps):
    # With a constant gradient g, bias-corrected moments are m_hat = g and v_hat = g^2 at
    # every step, so theta_{t+1} = a*theta_t - c with a = 1 - lr*wd, c = lr*g/(|g|+eps).
    # Exact rational recurrence; eps is large enough that sqrt(v_hat + eps) or
    # eps/sqrt(bias) variants would be far outside the tolerance.
    lr, b1, b2, wd = Fraction(1, 100), 0.8, 0.95, Fraction(1, 4)
    gq, epsq = Fraction(g0), Fraction(eps)
    a = 1 - lr * wd
    c = lr * gq / (abs(gq) + epsq)
    th = Fraction(3, 2)
    st = oracle.AdamWState([1.5], dtype=np.float64)
    for t in range(1, 21):
        th = a * th - c
        oracle.adamw_step(st, np.array([g0]), float(lr), b1, b2, eps, float(wd))
        assert st.theta[0] == pytest.approx(float(th), rel=1e-12), t
        assert st.m[0] == pytest.approx(g0 * (1 - b1 ** t), rel=1e-12)
        assert st.v[0] == pytest.approx(g0 * g0 * (1 - b2 ** t), rel=1e-12)


def test_first_step_is_sign_step():
    # t = 1, any g != 0: theta1 = theta*(1 - lr*wd) - lr*g/(|g| + eps).
    rng = np.random.default_rng(1)
    th = rng.normal(size=1000)
    g = rng.normal(size=1000) * 10.0 ** rng.integers(-6, 3, size=1000)
    st = oracle.AdamWState(th, dtype=np.float64)
    oracle.adamw_step(st, g, 1e-3, 0.9, 0.999, 1e-8, 0.1)
    want = th * (1 - 1e-3 * 0.1) - 1e-3 * g / (np.abs(g) + 1e-8)
    np.testing.assert_allclose(st.theta, want, rtol=1e-12, atol=0)


def test_zero_gradient_is_pure_decay():
    # g == 0 for H steps: theta_H = theta_0*(1 - lr*wd)^H, m = v = 0; and a zero element
    # (what padding holds) stays exactly zero.
    th = np.array([1.0, -2.5, 0.0, 1e-3], dtype=np.float64)
    st = oracle.AdamWState(th, dtype=np.float64)
    s32 = oracle.AdamWState(th)
    for _ in range(50):
        oracle.adamw_step(st, np.zeros(4), 4e-4, 0.9, 0.999, 1e-8, 0.1)
        oracle.adamw_step(s32, np.zeros(4, dtype=np.float32), 4e-4, 0.9, 0.999, 1e-8, 0.1)
    np.testing.assert_allclose(st.theta, th * (1 - 4e-5) ** 50, rtol=1e-13)
    np.testing.assert_allclose(s32.theta, th * (1 - 4e-5) ** 50, rtol=5e-6)
    assert not st.m.any() and not st.v.any()
    assert st.theta[2] == 0.0 and s32.theta[2] == 0.0
    assert not s32.m.any() and not s32.v.any()


@pytest.mark.parametrize("hp", [
    dict(lr=4e-4, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.1),
    dict(lr=3e-2, betas=(0.7, 0.93), eps=1e-3, weight_decay=0.3),
    dict(lr=1e-3, betas=(0.0, 0.5), eps=1e-6, weight_decay=0.0),
])
def test_against_library_adamw_float64(hp):
    # torch.optim.AdamW on CPU in float64: an independent implementation of the same
    # optimizer.  Both round differently, so agreement is to ~1e-12, which still
    # separates any formula difference (those are >= 1e-6).
    rng = np.random.default_rng(7)
    n, steps = 513, 25
    th0 = rng.normal(scale=0.02, size=n)
    th0[:7] = 1.0
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], foreach=False, **hp)
    st = oracle.AdamWState(th0, dtype=np.float64)
    for t in range(steps):
        g = rng.normal(scale=1e-3, size=n) * (1 + 10 * (t % 3))
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        oracle.adamw_step(st, g, hp["lr"], hp["betas"][0], hp["betas"][1], hp["eps"],
                          hp["weight_decay"])
        np.testing.assert_allclose(st.theta, p.detach().numpy(), rtol=2e-12, atol=1e-15)
    state = opt.state[p]
    np.testing.assert_allclose(st.m, state["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(st.v, state["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)


def test_float32_tracks_float64(paper_hp):
    # The float32 oracle (what the GPU is compared with) follows the float64 oracle to
    # float32 accuracy over a round of steps on the workload's value distributions.
    hp = paper_hp
    rng = np.random.default_rng(11)
    n = 4096
    th0 = rng.normal(scale=0.02, size=n).astype(np.float32)
    s32, s64 = oracle.AdamWState(th0), oracle.AdamWState(th0, dtype=np.float64)
    for _ in range(40):
        g = rng.normal(scale=1e-3, size=n).astype(np.float32)
        for st in (s32, s64):
            oracle.adamw_step(st, g, hp["inner_lr"], hp["beta1"], hp["beta2"], hp["eps"],
                              hp["weight_decay"])
    np.testing.assert_allclose(s32.theta, s64.theta, rtol=2e-5, atol=2e-7)
    np.testing.assert_allclose(s32.m, s64.m, rtol=1e-5, atol=1e-10)
    np.testing.assert_allclose(s32.v, s64.v, rtol=1e-5, atol=1e-13)


def test_elementwise_independence():
    # The value at index i depends on index i only: the oracle run on a subset of the
    # indices equals the subset of the oracle run on everything (bitwise).  This is what
    # licenses sampled parity at the large workloads.
    rng = np.random.default_rng(5)
    n = 10007
    idx = np.sort(rng.choice(n, size=300, replace=False))
    th0 = rng.normal(scale=0.02, size=n).astype(np.float32)
    full, sub = oracle.AdamWState(th0), oracle.AdamWState(th0[idx])
    for _ in range(6):
        g = rng.normal(scale=1e-3, size=n).astype(np.float32)
        oracle.adamw_step(full, g, 4e-4, 0.9, 0.999, 1e-8, 0.1)
        oracle.adamw_step(sub, g[idx], 4e-4, 0.9, 0.999, 1e-8, 0.1)
    assert np.array_equal(full.theta[idx], sub.theta)
    assert np.array_equal(full.m[idx], sub.m) and np.array_equal(full.v[idx], sub.v)


def test_unscale_is_widen_then_multiply():
    # binary16 gradients times 1/65536 (a power of two): exact, so the float64 product of
    # numpy's own widening is the expected value bit for bit.
    rng = np.random.default_rng(3)
    h = rng.normal(scale=65.0, size=5000).astype(np.float16)
    got = oracle.unscale_f16(h.view(np.uint16), 1.0 / 65536)
    want = (h.astype(np.float64) / 65536).astype(np.float32)
    assert np.array_equal(got, want)
    # A non power-of-two scale rounds once, in float32.
    got = oracle.unscale_f16(h.view(np.uint16), np.float32(1 / 3))
    want = (h.astype(np.float64) * float(np.float32(1 / 3))).astype(np.float32)
    assert np.array_equal(got, want)


def test_unscale_of_fp32_gradients():
    """The scaler's unscale also applies to gradients stored in FP32 ("General Implementation
    Details": the gradient scaler acts in the inner step).  A power-of-two loss scale is exact,
    so stepping (g * 2^16, inv_scale 2^-16) must equal stepping (g, no scale) bit for bit; a
    dropped multiply would change every element; hand values pin a non power-of-two factor."""
    rng = np.random.default_rng(11)
    n, k = 4099, 2
    th0 = rng.normal(scale=0.02, size=n).astype(np.float32)
    plain = oracle.DiLoCoOracle(th0, k, 4e-4, 0.9, 0.999, 1e-8, 0.1, 0.7, 0.9)
    scaled = oracle.DiLoCoOracle(th0, k, 4e-4, 0.9, 0.999, 1e-8, 0.1, 0.7, 0.9)
    for _ in range(3):
        g = [rng.normal(scale=1e-3, size=n).astype(np.float32) for _ in range(k)]
        plain.inner_step(g)
        scaled.inner_step([x * np.float32(65536) for x in g], inv_scale=2.0 ** -16)
    for a_, b_ in zip(plain.workers, scaled.workers):
        assert np.array_equal(a_.theta, b_.theta) and np.array_equal(a_.m, b_.m)
        assert np.array_equal(a_.v, b_.v)
    # without the factor the scaled gradients give a different result (the multiply is live)
    other = oracle.DiLoCoOracle(th0, k, 4e-4, 0.9, 0.999, 1e-8, 0.1, 0.7, 0.9)
    other.inner_step([x * np.float32(65536) for x in g])
    assert not np.array_equal(other.workers[0].m, plain.workers[0].m)
    # hand values: 3 * (1/3 rounded to float) rounds to exactly 1; 0.75 * 0.5 = 0.375; -2 * 0.25
    third = float(np.float32(1 / 3))
    assert oracle.unscale_f32(np.array([3.0], np.float32), third)[0] == np.float32(1.0)
    got = oracle.unscale_f32(np.array([0.75, -2.0, 0.0], np.float32), 0.5)
    assert got.tolist() == [0.375, -1.0, 0.0]
    assert oracle.unscale_f32(np.array([-2.0], np.float32), 0.25)[0] == np.float32(-0.5)


def test_skipped_worker_is_untouched():
    rng = np.random.default_rng(9)
    th0 = rng.normal(scale=0.02, size=257).astype(np.float32)
    o = oracle.DiLoCoOracle(th0, 3, 4e-4, 0.9, 0.999, 1e-8, 0.1, 0.7, 0.9)
    g = [rng.normal(scale=1e-3, size=257).astype(np.float32) for _ in range(3)]
    o.inner_step(g)
    before = [(w.theta.copy(), w.m.copy(), w.v.copy(), w.t, w.p1.value) for w in o.workers]
    o.inner_step(g, found_inf_flags=[0, 1, 0])
    w = o.workers[1]
    assert np.array_equal(w.theta, before[1][0]) and np.array_equal(w.m, before[1][1])
    assert np.array_equal(w.v, before[1][2]) and w.t == before[1][3] and w.p1.value == before[1][4]
    for r in (0, 2):
        assert o.workers[r].t == 2 and not np.array_equal(o.workers[r].theta, before[r][0])
    # The skipped worker's next step uses t = 2 (its own count), not the global call count.
    o.inner_step(g)
    assert o.workers[1].t == 2 and o.workers[0].t == 3
    assert o.workers[1].p1.value == pytest.approx(0.81, rel=1e-6)
