"""Pins for the oracle's flat-layout planner: brute-force properties on random size lists."""
import numpy as np

import oracle


def test_layout_properties_random_lists():
    rng = np.random.default_rng(0)
    for trial in range(200):
        nt = int(rng.integers(1, 40))
        numel = rng.integers(1, 5000, size=nt).astype(np.uint64)
        if trial % 3 == 0:
            numel[rng.integers(0, nt)] = 1
        align = int(rng.choice([1, 4, 64]))
        tile = int(rng.choice([64, 1024, 4096]))
        off, n_pad = oracle.plan_layout(numel, align, tile)
        assert off[0] == 0 and (off % align == 0).all()
        ends = off + numel
        assert (off[1:] >= ends[:-1]).all()                  # ascending, no overlap
        assert (off[1:] - ends[:-1] < align).all()           # no more padding than alignment needs
        assert n_pad % tile == 0 and n_pad >= ends[-1] and n_pad - int(ends[-1]) < tile


def test_scatter_gather_round_trip_and_zero_pads():
    rng = np.random.default_rng(1)
    numel = np.array([1, 63, 64, 65, 1000, 7], dtype=np.uint64)
    off, n_pad = oracle.plan_layout(numel, 64, 256)
    assert off.tolist() == [0, 64, 128, 192, 320, 1344] and n_pad == 1536
    tensors = [rng.normal(size=int(n)).astype(np.float32) for n in numel]
    flat = np.zeros(n_pad, dtype=np.float32)
    mask = np.zeros(n_pad, dtype=bool)
    for o, t in zip(off, tensors):
        flat[int(o):int(o) + t.size] = t
        assert not mask[int(o):int(o) + t.size].any()
        mask[int(o):int(o) + t.size] = True
    assert mask.sum() == numel.sum() and not flat[~mask].any()
    for o, t in zip(off, tensors):
        assert np.array_equal(flat[int(o):int(o) + t.size], t)
