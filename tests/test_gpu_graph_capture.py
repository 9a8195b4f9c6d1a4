"""Every entry point enqueues kernels only (no memset), and the per-worker step state is advanced
on the device by the step's own prologue kernel, so any number of inner steps -- odd counts
included -- can be captured into a HIP graph and replayed; every replay is checked against the
oracle, with eager work (outer steps and single inner steps) and synchronisations between the
replays."""
import numpy as np
import pytest

import synth
from harness import CpuSide, GpuSide, compare, compare_state

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_inner,layout_mode", [(2, 1), (3, 1), (3, 2)])
def test_captured_inner_steps_replay_correctly(n_inner, layout_mode):
    import torch
    wl = synth.tiny()
    k = 2
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gpu = GpuSide(wl, k, True, layout_mode=layout_mode)  # the context borrows the capturing stream
        g = gpu.gen_grads(0)
        flags = gpu.dl.new_flags()
    side.synchronize()
    cpu = CpuSide(wl, k, True)
    gc = cpu.gen_grads(0)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        gpu.dl.unscale_check(g, 1.0, flags)
        gpu.dl.inner_step(g, flags=flags)
        for _ in range(n_inner - 1):
            gpu.dl.inner_step(g)
    torch.cuda.synchronize()
    # capture itself executes nothing
    assert gpu.dl.steps() == [0, 0]

    total = 0
    for replay in range(4):
        graph.replay()
        torch.cuda.synchronize()
        cpu.o.inner_step(gc, found_inf_flags=[0, 0], inv_scale=1.0)
        for _ in range(n_inner - 1):
            cpu.o.inner_step(gc)
        total += n_inner
        assert compare_state(gpu, cpu, 0, 0) == 0, "replay %d" % replay
        assert flags.cpu().tolist() == [0, 0]
        # eager work of the same context between replays: an outer step, and on odd replays a
        # single eager inner step (an odd number of eager steps between two replays)
        with torch.cuda.stream(side):
            gpu.dl.outer_step()
            if replay % 2:
                gpu.dl.inner_step(g)
        side.synchronize()
        cpu.o.outer_step()
        if replay % 2:
            cpu.o.inner_step(gc)
            total += 1
        assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
        assert compare_state(gpu, cpu, 0, 0) == 0, "after eager work %d" % replay
    assert gpu.dl.steps() == [total, total]
    gpu.dl.close()
