"""Pins for the oracle's per-tensor parameter groups and learning-rate schedule: the grouped
step against separately stepped tensors (the already pinned single-group step), against
torch.optim.AdamW with param_groups in float64, and the schedule against hand values."""
import math

import numpy as np
import pytest
import torch

import oracle


def _layout(numel):
    off, n_pad = oracle.plan_layout(np.array(numel, dtype=np.uint64), 64, 256)
    return off, n_pad


def test_grouped_step_equals_separately_stepped_tensors():
    rng = np.random.default_rng(0)
    numel = [100, 64, 7, 300]
    off, n_pad = _layout(numel)
    grp = [0, 1, 1, 2]
    lr_scale, wd = [1.0, 0.5, 2.0], [0.1, 0.0, 0.3]
    G = oracle.ParamGroups(off, numel, grp, lr_scale, wd)
    th0 = np.zeros(n_pad, dtype=np.float32)
    for o, n in zip(off, numel):
        th0[int(o):int(o) + n] = rng.normal(scale=0.02, size=n)
    whole = oracle.AdamWState(th0)
    parts = [oracle.AdamWState(th0[int(o):int(o) + n]) for o, n in zip(off, numel)]
    for step in range(5):
        g = np.zeros(n_pad, dtype=np.float32)
        for o, n in zip(off, numel):
            g[int(o):int(o) + n] = rng.normal(scale=1e-3, size=n)
        oracle.adamw_step_groups(whole, g, G, 4e-4, 0.9, 0.999, 1e-8)
        for (o, n), t, st in zip(zip(off, numel), grp, parts):
            oracle.adamw_step(st, g[int(o):int(o) + n], 4e-4 * lr_scale[t], 0.9, 0.999, 1e-8, wd[t])
    for (o, n), st in zip(zip(off, numel), parts):
        sl = slice(int(o), int(o) + n)
        assert np.array_equal(whole.theta[sl], st.theta)
        assert np.array_equal(whole.m[sl], st.m) and np.array_equal(whole.v[sl], st.v)
    pad = np.ones(n_pad, dtype=bool)
    for o, n in zip(off, numel):
        pad[int(o):int(o) + n] = False
    assert not whole.theta[pad].any() and not whole.m[pad].any()
    assert whole.t == 5 and whole.p1.value == pytest.approx(0.9 ** 5, rel=1e-14)


def test_grouped_step_against_library_param_groups_float64():
    rng = np.random.default_rng(1)
    numel = [50, 128, 9]
    off, n_pad = _layout(numel)
    grp, lr_scale, wd = [0, 1, 0], [1.0, 0.25], [0.1, 0.0]
    G = oracle.ParamGroups(off, numel, grp, lr_scale, wd)
    th0 = rng.normal(scale=0.02, size=n_pad)
    ps = [torch.nn.Parameter(torch.tensor(th0[int(o):int(o) + n])) for o, n in zip(off, numel)]
    opt = torch.optim.AdamW([dict(params=[ps[0], ps[2]], lr=3e-3, weight_decay=0.1),
                             dict(params=[ps[1]], lr=3e-3 * 0.25, weight_decay=0.0)],
                            betas=(0.9, 0.95), eps=1e-6, foreach=False)
    st = oracle.AdamWState(th0, dtype=np.float64)
    for _ in range(10):
        g = rng.normal(scale=1e-2, size=n_pad)
        for p, (o, n) in zip(ps, zip(off, numel)):
            p.grad = torch.tensor(g[int(o):int(o) + n])
        opt.step()
        oracle.adamw_step_groups(st, g, G, 3e-3, 0.9, 0.95, 1e-6)
    for p, (o, n) in zip(ps, zip(off, numel)):
        np.testing.assert_allclose(st.theta[int(o):int(o) + n], p.detach().numpy(), rtol=2e-12)


def test_lr_schedule_hand_values():
    # warm-up: linear from 0; the paper trains with 1000 warm-up steps and base rate 4e-4
    assert oracle.lr_at(0, 1000, 0, 4e-4) == 0.0
    assert oracle.lr_at(250, 1000, 0, 4e-4) == pytest.approx(1e-4, rel=1e-15)
    assert oracle.lr_at(999, 1000, 0, 4e-4) == pytest.approx(4e-4 * 0.999, rel=1e-15)
    assert oracle.lr_at(1000, 1000, 0, 4e-4) == 4e-4
    assert oracle.lr_at(10 ** 9, 1000, 0, 4e-4) == 4e-4            # no decay requested
    # cosine decay to 10 % between step 1000 and 88000
    assert oracle.lr_at(1000, 1000, 88000, 4e-4, 0.1) == pytest.approx(4e-4, rel=1e-15)
    mid = 1000 + (88000 - 1000) // 2
    want = 4e-4 * (0.1 + 0.9 * 0.5 * (1 + math.cos(math.pi * (mid - 1000) / 87000)))
    assert oracle.lr_at(mid, 1000, 88000, 4e-4, 0.1) == pytest.approx(want, rel=1e-14)
    assert oracle.lr_at(44500, 1000, 88000, 4e-4, 0.0) == pytest.approx(2e-4, rel=1e-12)
    assert oracle.lr_at(88000, 1000, 88000, 4e-4, 0.1) == pytest.approx(4e-5, rel=1e-15)
    assert oracle.lr_at(99999, 1000, 88000, 4e-4, 0.1) == pytest.approx(4e-5, rel=1e-15)
    # monotone: up during warm-up, down afterwards
    xs = [oracle.lr_at(s, 100, 1000, 1.0, 0.0) for s in range(0, 1001, 10)]
    assert all(b >= a for a, b in zip(xs[:10], xs[1:11])) and all(b <= a for a, b in zip(xs[10:], xs[11:]))
