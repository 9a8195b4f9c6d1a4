"""Mixed-precision stress: the 150M set plus 2000 ragged tiny tensors, k=4, binary16 gradients
pre-scaled by 65536, 0.01 % of one worker's elements inf/NaN.  The inf check must flag exactly
that worker, its inner step must be skipped bit for bit, and the others must match the oracle."""
import numpy as np
import pytest

import oracle
import synth
from harness import CpuSide, GpuSide, compare, compare_state

pytestmark = pytest.mark.gpu

INV_SCALE = 1.0 / 65536


@pytest.mark.timeout(900)
def test_stress_unscale_check_and_skip():
    wl = synth.stress()
    assert len(wl.shapes) == 2109
    k, bad = 4, 2
    gpu, cpu = GpuSide(wl, k), CpuSide(wl, k)
    assert gpu.n_pad == cpu.n_pad and list(gpu.dl.offsets) == [int(o) for o in cpu.offsets]
    flags = gpu.dl.new_flags()
    flags.fill_(7)                                    # stale content must be overwritten

    # step 0: worker `bad` has non-finite gradients
    g = gpu.gen_grads(0, f16=True, inject_replica=bad, inject_period=10000)
    gc = cpu.gen_grads(0, f16=True, inject_replica=bad, inject_period=10000)
    for r in range(k):
        assert np.array_equal(gpu.host(g[r].view(gpu.torch.int16)).view(np.uint16), gc[r])
    want_flags = [oracle.found_inf(x) for x in gc]
    assert want_flags == [0, 0, 1, 0]
    n_bad = int(((gc[bad] & 0x7C00) == 0x7C00).sum())
    assert 0.5e-4 * wl.n_params < n_bad < 2e-4 * wl.n_params
    gpu.dl.unscale_check(g, INV_SCALE, flags)
    assert flags.cpu().tolist() == want_flags
    before = [gpu.host(t[bad]).copy() for t in (gpu.dl.theta, gpu.dl.m, gpu.dl.v)]
    gpu.dl.inner_step(g, flags=flags)
    cpu.o.inner_step(gc, found_inf_flags=want_flags, inv_scale=INV_SCALE)
    assert gpu.dl.steps() == [1, 1, 0, 1]
    for t, b in zip((gpu.dl.theta, gpu.dl.m, gpu.dl.v), before):
        assert np.array_equal(gpu.host(t[bad]).view(np.uint32), b.view(np.uint32))
    assert compare_state(gpu, cpu) == 0

    # step 1: clean gradients; the skipped worker now takes ITS first step (t = 1)
    g = gpu.gen_grads(1, f16=True)
    gc = cpu.gen_grads(1, f16=True)
    gpu.dl.unscale_check(g, INV_SCALE, flags)
    assert flags.cpu().tolist() == [0, 0, 0, 0]
    gpu.dl.inner_step(g, flags=flags)
    cpu.o.inner_step(gc, found_inf_flags=[0] * k, inv_scale=INV_SCALE)
    assert gpu.dl.steps() == [2, 2, 1, 2] and [w.t for w in cpu.o.workers] == [2, 2, 1, 2]
    assert compare_state(gpu, cpu) == 0
    # the outer step never looks at flags or scale
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 1e-5, 1e-7) == 0
    assert flags.cpu().tolist() == [0, 0, 0, 0]
    gpu.dl.close()


@pytest.mark.parametrize("layout_mode", [1, 2])
def test_flag_positions_brute_force(layout_mode):
    """One special value at chosen positions of small ragged tensor lists: first/last element of
    a tensor, element before a pad, last real element; both gradient types."""
    torch = pytest.importorskip("torch")
    import paper_2407_07852_amd as D
    numel = [1, 63, 64, 65, 4096, 7, 1000]
    k = 3
    dl = D.DiLoCo(numel, k, fill_theta0=lambda t, lay, off: t.zero_(), layout_mode=layout_mode)
    flags = dl.new_flags()
    positions = []
    for off, n in zip(dl.offsets, numel):
        positions += [off, off + n - 1, off + n // 2]
    for dtype, specials in ((torch.float16, [(float("inf"), 1), (float("-inf"), 1), (float("nan"), 1),
                                             (65504.0, 0), (-65504.0, 0), (6e-8, 0)]),
                            (torch.float32, [(float("inf"), 1), (float("nan"), 1), (3.4e38, 0),
                                             (1e-45, 0)])):
        g = dl.new_grads(dtype)
        for r in range(k):
            for pos in sorted(set(positions)):
                for val, want in specials:
                    g.zero_()
                    g[r, pos] = val
                    dl.unscale_check(g, 1.0, flags)
                    expect = [0] * k
                    expect[r] = want
                    assert flags.cpu().tolist() == expect, (dtype, r, pos, val)
                    host = g[r].cpu()
                    bits = host.view(torch.int16).numpy().view(np.uint16) if dtype == torch.float16 \
                        else host.numpy()
                    assert oracle.found_inf(bits) == want
    dl.close()
