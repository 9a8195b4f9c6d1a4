"""Pins for the oracle's outer step: pseudo-gradient sign, worker average (order and
divisor), Nesterov convention, reset/broadcast; against hand-computed values, exact
rational arithmetic, numpy reductions and the PyTorch wheel's SGD in float64."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle


def test_pseudo_gradient_sign():
    # Original minus locally updated weight (Section "Implementation").
    d = oracle.pseudo_grad(np.array([1.0, -2.0], dtype=np.float32),
                           np.array([0.75, -2.5], dtype=np.float32))
    assert d.tolist() == [0.25, 0.5]


def test_nesterov_by_hand(paper_hp):
    # theta=1, b=0, mu=0.9, lr=0.7, grad 0.1 twice:
    #   b1 = 0.1,  theta1 = 1 - 0.7*(0.1 + 0.09)   = 0.867
    #   b2 = 0.19, theta2 = 0.867 - 0.7*(0.1+0.171) = 0.6773
    th, b, g = np.array([1.0]), np.array([0.0]), np.array([0.1])
    oracle.nesterov_step(th, b, g, paper_hp["outer_lr"], paper_hp["outer_momentum"])
    assert b[0] == pytest.approx(0.1, rel=1e-15) and th[0] == pytest.approx(0.867, rel=1e-14)
    oracle.nesterov_step(th, b, g, paper_hp["outer_lr"], paper_hp["outer_momentum"])
    assert b[0] == pytest.approx(0.19, rel=1e-14) and th[0] == pytest.approx(0.6773, rel=1e-14)


def test_nesterov_zero_momentum_is_plain_sgd():
    rng = np.random.default_rng(2)
    th0, g = rng.normal(size=100), rng.normal(size=100)
    th, b = th0.copy(), rng.normal(size=100)
    oracle.nesterov_step(th, b, g, 0.7, 0.0)
    np.testing.assert_allclose(th, th0 - 0.7 * g, rtol=1e-15)
    np.testing.assert_array_equal(b, g)


@pytest.mark.parametrize("lr,mu", [(0.7, 0.9), (0.05, 0.5), (1.0, 0.99)])
def test_nesterov_against_library_sgd_float64(lr, mu):
    rng = np.random.default_rng(4)
    n = 300
    th0 = rng.normal(size=n)
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True, foreach=False)
    th, b = th0.copy(), np.zeros(n)
    for _ in range(12):
        g = rng.normal(scale=0.01, size=n)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        oracle.nesterov_step(th, b, g, lr, mu)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(b, opt.state[p]["momentum_buffer"].numpy(), rtol=1e-13, atol=1e-18)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8])
def test_mean_of_identical_replicas_is_each_delta(k):
    rng = np.random.default_rng(k)
    d = rng.normal(scale=1e-2, size=1000).astype(np.float32)
    d[:3] = [0.0, 6e-8, -1e-40]     # zero, subnormal half range, subnormal float
    mean = oracle.replica_mean(np.tile(d, (k, 1)))
    if k in (1, 2, 4):
        # d+d is exact, (2d+d) can only miss by a tie that the next addition repairs, and
        # dividing by a power of two is exact: the mean is each delta, bitwise.
        assert np.array_equal(mean.view(np.uint32), d.view(np.uint32))
    else:
        # Partial sums 3d, 5d, ... need more significand bits than a float has, so the
        # sequential sum rounds; the mean is each delta to within the k-1 roundings.
        assert (np.abs(mean.astype(np.float64) - d) <= k * 2.0 ** -24 * np.abs(d)).all()
    # Values on a coarse grid (20-bit integers) make every partial sum exact for any k.
    q = rng.integers(-2 ** 20, 2 ** 20, size=1000).astype(np.float32)
    mean = oracle.replica_mean(np.tile(q, (k, 1)))
    want = (q.astype(np.float64) * k / k).astype(np.float32) if k in (1, 2, 4, 8) else None
    if want is not None:
        assert np.array_equal(mean, want)


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
def test_mean_against_exact_rational(k):
    rng = np.random.default_rng(10 + k)
    d = rng.normal(scale=1e-2, size=(k, 200)).astype(np.float32)
    mean = oracle.replica_mean(d)
    for i in range(200):
        exact = sum(Fraction(float(x)) for x in d[:, i]) / k
        # k-1 additions and a division, each within half an ulp of its own result.
        tol = (k + 1) * 2.0 ** -24 * max(abs(float(x)) for x in d[:, i])
        assert abs(Fraction(float(mean[i])) - exact) <= tol
    m64 = oracle.replica_mean(d.astype(np.float64))
    np.testing.assert_allclose(m64, d.astype(np.float64).mean(axis=0), rtol=1e-13, atol=1e-18)


def test_mean_sums_in_worker_order():
    # (1e8 + 1) rounds to 1e8 in float32, so worker order 0,1,2 gives exactly 0;
    # any order that adds 1e8 and -1e8 first would give 1/3.
    d = np.array([[1e8], [1.0], [-1e8]], dtype=np.float32)
    assert oracle.replica_mean(d)[0] == 0.0
    d = np.array([[1e8], [-1e8], [1.0]], dtype=np.float32)
    assert oracle.replica_mean(d)[0] == np.float32(1.0) / np.float32(3.0)


def test_outer_step_with_no_inner_steps_is_momentum_decay_only():
    # H = 0: every worker still equals theta0, so every pseudo-gradient is +0 and only the
    # momentum acts.  b=1, mu=0.5, lr=0.25, theta0=2: b' = 0.5, theta0' = 2 - 0.25*0.25.
    th0 = np.full(5, 2.0, dtype=np.float32)
    b = np.ones(5, dtype=np.float32)
    theta = np.tile(th0, (4, 1))
    mean = oracle.outer_step(th0, b, theta, 0.25, 0.5, False)
    assert not mean.any() and not np.signbit(mean).any()
    assert (b == 0.5).all() and (th0 == 1.9375).all() and (theta == 1.9375).all()
    # ... and with b = 0 it is the identity.
    th0 = np.full(5, 2.0, dtype=np.float32)
    b = np.zeros(5, dtype=np.float32)
    theta = np.tile(th0, (4, 1))
    oracle.outer_step(th0, b, theta, 0.7, 0.9, True)
    assert (th0 == 2.0).all() and (b == 0.0).all() and (theta == 2.0).all()


def test_unit_lr_zero_momentum_is_parameter_averaging():
    # lr = 1, mu = 0: theta0' = theta0 - mean(theta0 - theta_r) = mean_r(theta_r) up to
    # rounding; every worker is reset to it.
    rng = np.random.default_rng(6)
    k, n = 4, 500
    th0 = rng.normal(scale=0.02, size=n).astype(np.float32)
    theta = (th0 + rng.normal(scale=1e-3, size=(k, n))).astype(np.float32)
    want = theta.astype(np.float64).mean(axis=0)
    b = np.zeros(n, dtype=np.float32)
    oracle.outer_step(th0, b, theta, 1.0, 0.0, False)
    np.testing.assert_allclose(th0, want, rtol=0, atol=2e-8)
    for r in range(k):
        assert np.array_equal(theta[r], th0)


def test_outer_step_composition_by_hand():
    # k=2, theta0=1, workers 0.5 and 0.75, b=0.25, mu=0.5, lr=0.5 (all exact in binary):
    # deltas 0.5, 0.25 -> mean 0.375 ; b' = 0.125+0.375 = 0.5 ;
    # theta0' = 1 - 0.5*(0.375 + 0.25) = 0.6875.
    th0 = np.array([1.0], dtype=np.float32)
    b = np.array([0.25], dtype=np.float32)
    theta = np.array([[0.5], [0.75]], dtype=np.float32)
    mean = oracle.outer_step(th0, b, theta, 0.5, 0.5, False)
    assert mean[0] == 0.375 and b[0] == 0.5 and th0[0] == 0.6875
    assert theta.tolist() == [[0.6875], [0.6875]]


def test_fp16_pseudo_gradient_rounds_each_worker_before_the_mean():
    # delta_0 = 1 + 2^-11 (a tie: rounds to 1.0 in binary16), delta_1 = 1 + 3*2^-11
    # (rounds to 1 + 2^-9).  Rounding each worker first gives mean 1 + 2^-10; rounding
    # the mean instead would give 1 + 2^-10 as well only by accident of ties, so use a
    # third case: delta = 2^-25 (flushes to 0 in binary16 by ties-to-even).
    th0 = np.zeros(3, dtype=np.float32)
    theta = -np.array([[1 + 2.0 ** -11, 2.0 ** -25, 70000.0],
                       [1 + 3 * 2.0 ** -11, 2.0 ** -25, 0.0]], dtype=np.float32)
    b = np.zeros(3, dtype=np.float32)
    mean = oracle.outer_step(th0, b, theta.copy(), 1.0, 0.0, True)
    assert mean[0] == np.float32(1 + 2.0 ** -10)
    assert mean[1] == 0.0                       # each 2^-25 became 0 before the sum
    assert np.isinf(mean[2]) and mean[2] > 0    # 70000 overflows binary16
    mean32 = oracle.outer_step(np.zeros(3, dtype=np.float32), np.zeros(3, dtype=np.float32),
                               theta.copy(), 1.0, 0.0, False)
    assert mean32[1] == np.float32(2.0 ** -25) and mean32[2] == 35000.0


def test_outer_step_does_not_touch_inner_state():
    rng = np.random.default_rng(8)
    th0 = rng.normal(scale=0.02, size=100).astype(np.float32)
    o = oracle.DiLoCoOracle(th0, 2, 4e-4, 0.9, 0.999, 1e-8, 0.1, 0.7, 0.9)
    for _ in range(3):
        o.inner_step([rng.normal(scale=1e-3, size=100).astype(np.float32) for _ in range(2)])
    snap = [(w.m.copy(), w.v.copy(), w.t, w.p1.value, w.p2.value) for w in o.workers]
    o.outer_step()
    for w, s in zip(o.workers, snap):
        assert np.array_equal(w.m, s[0]) and np.array_equal(w.v, s[1])
        assert (w.t, w.p1.value, w.p2.value) == s[2:]
        assert np.array_equal(w.theta, o.theta0)
