"""Pins of the delayed application of the outer step (the paper's Conclusion names asynchronous
weight averaging interleaved with the next round's computation as future work and gives no
rule; the rule taken: the outer update is computed from snapshots sigma_r of the workers'
weights, and applied later as theta_r <- theta0_new - (sigma_r - theta_r))."""
import numpy as np
import pytest

import oracle

HP = (4e-4, 0.9, 0.999, 1e-8, 0.1)


def make(k=3, n=4099, seed=0, pg=False, rm=False):
    rng = np.random.default_rng(seed)
    th0 = rng.normal(scale=0.02, size=n).astype(np.float32)
    th0[::97] = -0.0                                     # signed zeros must survive
    o = oracle.DiLoCoOracle(th0, k, *HP, 0.7, 0.9, pg, rm)
    return o, rng


def inner(o, rng, steps):
    n = o.theta0.size
    for _ in range(steps):
        o.inner_step([rng.normal(scale=1e-3, size=n).astype(np.float32) for _ in range(o.k)])


@pytest.mark.parametrize("pg,rm", [(False, False), (True, False), (oracle.PG_BF16, True)])
def test_no_steps_in_between_is_the_outer_step_of_figure_1(pg, rm):
    a, rng_a = make(pg=pg, rm=rm)
    b, rng_b = make(pg=pg, rm=rm)
    for rnd in range(2):                                  # second round: momentum is live
        inner(a, rng_a, 3)
        inner(b, rng_b, 3)
        a.outer_step()
        b.outer_begin()
        b.outer_finish()
        assert np.array_equal(a.theta0.view(np.uint32), b.theta0.view(np.uint32))
        assert np.array_equal(a.b.view(np.uint32), b.b.view(np.uint32))
        for wa, wb in zip(a.workers, b.workers):
            assert np.array_equal(wa.theta.view(np.uint32), wb.theta.view(np.uint32))
            assert np.array_equal(wa.m, wb.m) and wa.t == wb.t


def test_one_element_by_hand():
    # theta0 = 1, snapshot 0.9, the worker has moved on to 0.85 when the update is applied;
    # k = 1, b = 0, mu = 0.9, eta = 0.7:  delta = 0.1, b = 0.1,
    # theta0' = 1 - 0.7*(0.1 + 0.09) = 0.867;  theta = 0.867 - (0.9 - 0.85) = 0.817
    th0, b = np.array([1.0], np.float32), np.zeros(1, np.float32)
    snap = np.array([[0.9]], np.float32)
    mean = oracle.outer_update_from_snapshot(th0, b, snap, 0.7, 0.9)
    assert mean[0] == pytest.approx(0.1, rel=1e-6) and b[0] == pytest.approx(0.1, rel=1e-6)
    assert th0[0] == pytest.approx(0.867, rel=1e-6)
    theta = np.array([[0.85]], np.float32)
    oracle.merge_delayed(th0, snap, theta)
    assert theta[0, 0] == pytest.approx(0.817, rel=1e-6)
    # the same in double, to the last digits
    th0d, snapd, thetad = np.array([0.867]), np.array([[0.9]]), np.array([[0.85]])
    oracle.merge_delayed(th0d, snapd, thetad)
    assert thetad[0, 0] == pytest.approx(0.817, rel=1e-15)
    # progress in the other direction has the other sign
    thetad = np.array([[0.95]])
    oracle.merge_delayed(th0d, snapd, thetad)
    assert thetad[0, 0] == pytest.approx(0.917, rel=1e-15)


def test_progress_since_the_snapshot_is_carried_over_exactly():
    """Values on a coarse binary grid, so that every operation is exact: afterwards each worker
    sits at theta0_new + (theta_r - sigma_r), whatever the snapshots were."""
    rng = np.random.default_rng(4)
    k, n = 4, 1000
    grid = lambda size: (rng.integers(-512, 512, size=size) / 1024.0)
    th0 = grid(n)
    snap = grid((k, n))
    progress = grid((k, n))
    theta = snap + progress
    for dt in (np.float64, np.float32):
        t0, s, t = th0.astype(dt), snap.astype(dt), theta.astype(dt)
        oracle.merge_delayed(t0, s, t)
        assert np.array_equal(t, (th0 + progress).astype(dt))


def test_update_from_snapshot_reads_the_snapshots_not_the_workers():
    o, rng = make(k=2, n=515)
    inner(o, rng, 2)
    ref, _ = make(k=2, n=515)
    ref_rng = np.random.default_rng(0)
    ref_rng.normal(scale=0.02, size=515)                  # same stream as make()
    inner(ref, ref_rng, 2)
    o.outer_begin()
    inner(o, rng, 2)                                      # the workers move on; theta0, b must not care
    th0_after_begin, b_after_begin = o.theta0.copy(), o.b.copy()
    ref.outer_step()
    assert np.array_equal(th0_after_begin, ref.theta0) and np.array_equal(b_after_begin, ref.b)
    before = [w.theta.copy() for w in o.workers]
    snap = o.snap.copy()
    o.outer_finish()
    for r, w in enumerate(o.workers):
        want = (o.theta0 - (snap[r] - before[r])).astype(np.float32)
        assert np.array_equal(w.theta, want)
        assert not np.array_equal(w.theta, o.theta0)      # the progress is really there
